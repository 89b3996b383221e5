// Sampling and verification kernels that follow the vocabulary head (Algorithm 2 of the
// paper, lines "Sample draft tokens" to "break", and the LowConf re-corruption):
//
//   row_lse_draft_kernel     one wavefront per logits row: merge the head kernel's per-tile
//                            (max, sum exp) partials into the row's log-sum-exp; draft rows
//                            also locate their window slot and draw x~ ~ rho by a two-level
//                            inverse CDF (tiles, then tokens inside the tile).
//   accept_resid_kernel      per sequence: accept tests u <= min{1, pi(x~)/rho(x~)}, first
//                            rejection by ballot; per 256-token chunk the residual mass
//                            sum [pi - rho]_+ (and the overlap mass sum min{pi, rho}) of the
//                            rejected slot.
//   finalize_kernel          per sequence: inverse CDF over the residual chunks and inside
//                            the selected chunk, commit of tokens and confidences, block-mask
//                            update and LowConf.  (A separate launch on purpose: handing the
//                            chunk masses to a last-arriving workgroup inside one kernel needs
//                            device-scope fences, which write back and invalidate a whole
//                            XCD's L2 each time; measured 300 us at B = 64 against 13 us.)
//
// Every floating-point reduction uses a fixed tree (no float atomics), so results are
// reproducible bit for bit.
#include <limits.h>
#include <math.h>

#include "fef_device.hpp"
#include "wave_ops.hpp"

namespace fef {
namespace {

constexpr int NT = 256;          // threads per workgroup of every kernel in this file
constexpr int NW = NT / kWave;   // wavefronts per workgroup

struct BlockTmp {
  float f[NW];
  int i[NW];
  float bcast_f;
  int bcast_i;
};

__device__ inline float block_sum(float x, BlockTmp& t) {
  x = wave_sum(x);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) t.f[threadIdx.x >> 6] = x;
  __syncthreads();
  float s = 0.f;
#pragma unroll
  for (int w = 0; w < NW; ++w) s += t.f[w];
  return s;
}
__device__ inline float block_max(float x, BlockTmp& t) {
  x = wave_max(x);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) t.f[threadIdx.x >> 6] = x;
  __syncthreads();
  float s = t.f[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) s = fmaxf(s, t.f[w]);
  return s;
}
__device__ inline int block_min_int(int x, BlockTmp& t) {
  x = wave_min_int(x);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) t.i[threadIdx.x >> 6] = x;
  __syncthreads();
  int s = t.i[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) s = min(s, t.i[w]);
  return s;
}
__device__ inline int block_max_int(int x, BlockTmp& t) {
  x = wave_max_int(x);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) t.i[threadIdx.x >> 6] = x;
  __syncthreads();
  int s = t.i[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) s = max(s, t.i[w]);
  return s;
}

// Exclusive prefix sum of one value per thread in thread order; `total` gets the sum.
__device__ inline float block_exclusive_scan(float x, BlockTmp& t, float& total) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const float inc = wave_scan_add(x);
  float exc = __shfl_up(inc, 1, 64);
  if (lane == 0) exc = 0.f;
  __syncthreads();
  if (lane == 63) t.f[w] = inc;
  __syncthreads();
  float base = 0.f, tot = 0.f;
#pragma unroll
  for (int i = 0; i < NW; ++i) {
    if (i == w) base = tot;
    tot += t.f[i];
  }
  total = tot;
  return base + exc;
}

struct Found {
  int idx;       // first index whose inclusive prefix sum reaches the target
  float before;  // prefix sum of everything before idx
  float total;   // sum of all masses
};

// min{i in [0,n) : sum_{j<=i} mass(j) >= target} over non-negative masses, ascending i.
// Thread t owns the contiguous segment [t*per, (t+1)*per).  If rounding leaves every prefix
// below the target, the last index with positive mass is returned (index 0 if there is none).
template <class F>
__device__ inline Found block_find_first(int n, F mass, float target, BlockTmp& t) {
  const int per = (n + NT - 1) / NT;
  const int begin = min(n, (int)threadIdx.x * per), end = min(n, begin + per);
  float local = 0.f;
  for (int i = begin; i < end; ++i) local += mass(i);
  float total;
  const float exc = block_exclusive_scan(local, t, total);
  float run = exc, before = 0.f, before_pos = 0.f;
  int cand = INT_MAX, last_pos = -1;
  for (int i = begin; i < end; ++i) {
    const float mi = mass(i);
    const float nxt = run + mi;
    if (mi > 0.f) { last_pos = i; before_pos = run; }
    if (cand == INT_MAX && nxt >= target) { cand = i; before = run; }
    run = nxt;
  }
  int win = block_min_int(cand, t);
  bool mine = cand != INT_MAX && cand == win;
  if (win == INT_MAX) {  // target not reached: fall back to the last positive mass
    const int lp = block_max_int(last_pos, t);
    if (lp < 0) { win = 0; mine = threadIdx.x == 0; before = 0.f; }
    else { win = lp; mine = last_pos == lp; before = before_pos; }
  }
  __syncthreads();
  if (mine) t.bcast_f = before;
  __syncthreads();
  Found f;
  f.idx = win;
  f.before = t.bcast_f;
  f.total = total;
  return f;
}

// Token range of partial tile i: [unit * floor(i T / G), unit * floor((i+1) T / G)) within [0, V).
__device__ inline int tile_start(const VerifyArgs& a, int i) {
  return (int)((long)i * a.tile_T / a.tile_G) * a.tile_unit;
}

// Wavefront version of block_find_first: lane l owns the contiguous segment [l*per, (l+1)*per).
template <class F>
__device__ inline Found wave_find_first(int n, F mass, float target) {
  const int lane = threadIdx.x & 63;
  const int per = (n + kWave - 1) / kWave;
  const int begin = min(n, lane * per), end = min(n, begin + per);
  float local = 0.f;
  for (int i = begin; i < end; ++i) local += mass(i);
  const float inc = wave_scan_add(local);
  float exc = __shfl_up(inc, 1, 64);
  if (lane == 0) exc = 0.f;
  float run = exc, before = 0.f, before_pos = 0.f;
  int cand = INT_MAX, last_pos = -1;
  for (int i = begin; i < end; ++i) {
    const float mi = mass(i);
    const float nxt = run + mi;
    if (mi > 0.f) { last_pos = i; before_pos = run; }
    if (cand == INT_MAX && nxt >= target) { cand = i; before = run; }
    run = nxt;
  }
  int win = wave_min_int(cand);
  bool mine = cand != INT_MAX && cand == win;
  if (win == INT_MAX) {  // target not reached: fall back to the last positive mass
    const int lp = wave_max_int(last_pos);
    if (lp < 0) { win = 0; mine = lane == 0; before = 0.f; }
    else { win = lp; mine = last_pos == lp; before = before_pos; }
  }
  const unsigned long long owner = __ballot(mine);
  Found f;
  f.idx = win;
  f.before = __shfl(before, __ffsll((long long)owner) - 1, 64);
  f.total = __shfl(inc, 63, 64);
  return f;
}

// Register-resident variant of wave_find_first: lane l holds the masses of elements
// l*PER .. l*PER + PER-1 (zero beyond the end).
// REL: the target is a fraction of the total mass.
template <int PER, bool REL = false>
__device__ inline Found wave_find_first_reg(const float (&m)[PER], float target) {
  const int lane = threadIdx.x & 63;
  float local = 0.f;
#pragma unroll
  for (int j = 0; j < PER; ++j) local += m[j];
  const float inc = wave_scan_add(local);
  if (REL) target *= __shfl(inc, 63, 64);
  float exc = __shfl_up(inc, 1, 64);
  if (lane == 0) exc = 0.f;
  float run = exc, before = 0.f, before_pos = 0.f;
  int cand = -1, last_pos = -1;
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    const float nxt = run + m[j];
    if (m[j] > 0.f) { last_pos = j; before_pos = run; }
    if (cand < 0 && nxt >= target) { cand = j; before = run; }
    run = nxt;
  }
  // segments ascend with the lane id: the lowest lane that reached the target holds the answer
  unsigned long long hit = __ballot(cand >= 0);
  int owner;
  if (hit) {
    owner = __ffsll((long long)hit) - 1;
  } else {  // target not reached: fall back to the last positive mass
    hit = __ballot(last_pos >= 0);
    owner = hit ? 63 - __clzll((long long)hit) : 0;
    cand = last_pos < 0 ? 0 : last_pos;
    before = before_pos;
  }
  Found f;
  f.idx = owner * PER + __shfl(cand, owner, 64);
  f.before = __shfl(before, owner, 64);
  f.total = __shfl(inc, 63, 64);
  return f;
}

// window slot m = (m+1)-th unresolved position of block b in ascending order; also counts the
// unresolved positions.  Whole wavefront.
__device__ inline int window_slot(const VerifyArgs& a, int b, int m, int& unresolved) {
  const int lane = threadIdx.x & 63;
  int cnt = 0, pos = -1;
  for (int base = 0; base < a.block; base += kWave) {
    const int i = base + lane;
    const bool bit = i < a.block && (a.mask_in ? a.mask_in[(size_t)b * a.block + i] != 0 : true);
    const unsigned long long bal = __ballot(bit);
    const int rank = cnt + __popcll(bal & ((1ull << lane) - 1ull));
    if (bit && rank == m) pos = i;
    cnt += __popcll(bal);
  }
  unresolved = cnt;
  return wave_max_int(pos);
}

// Greedy variant: arg max of a logits row (lowest token id on a tie) from the head kernel's
// partials.  Every partial maximum is the exact maximum of the stored logits of its tile, so the
// first tile whose maximum equals the row maximum holds the answer, and the first token of that
// tile whose stored logit equals it is the arg max.  Whole wavefront.
__device__ inline int row_argmax(const VerifyArgs& a, const float2* P, const float* L, float row_max) {
  const int lane = threadIdx.x & 63;
  int cand = INT_MAX;
  for (int t = lane; t < a.nT && cand == INT_MAX; t += kWave)
    if (P[t].x == row_max) cand = t;
  const int tile = wave_min_int(cand);
  if (tile == INT_MAX) return 0;  // only if the row holds NaN
  const int v0 = tile_start(a, tile);
  const int nv = min(tile_start(a, tile + 1), a.V) - v0;
  cand = INT_MAX;
  for (int i = lane; i < nv && cand == INT_MAX; i += kWave)
    if (L[v0 + i] == row_max) cand = i;
  const int idx = wave_min_int(cand);
  return idx == INT_MAX ? v0 : v0 + idx;
}

constexpr int kChunkPer = 16;  // residual chunks per lane in the one-wavefront final phase
constexpr int kTilePer = 10;  // tokens per lane inside one partial tile: tiles of up to 640 tokens (a 151936-token
                              // vocabulary over 256 workgroups: 576 to 640 tokens each), longer ones are re-read

// ---------------------------------------------------------------------------------------------
// Kernel 1: per-row log-sum-exp, window slot, draft sample.  One wavefront per row.
// PER > 0: the row's partials (at most 64*PER) and the tokens of the selected tile live in
// registers, so every global value is loaded once and every exponential evaluated once.
// PER == 0: any number of partials, re-read from memory.
// ---------------------------------------------------------------------------------------------
template <int PER>
__global__ __launch_bounds__(NT) void row_lse_draft_kernel(VerifyArgs a) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int BK = a.B * a.K;
  const int r = a.row0 + blockIdx.x * NW + wave;
  if (r >= a.row0 + a.nrows) return;
  const bool is_draft = r < BK;
  const int s = is_draft ? r : r - BK;
  const int b = s / a.K, m = s % a.K;
  const float2* P = a.partials + (size_t)r * a.nT;

  // log-sum-exp of the row from the head kernel's per-tile partials
  float mass[PER > 0 ? PER : 1];  // exp-sums of this lane's tiles relative to the row maximum
  float mx = -INFINITY, sm = 0.f;
  if constexpr (PER > 0) {
    // Lane l owns the consecutive tiles l*PER .. l*PER + PER-1 (the ordered search below needs
    // that).  With few partials per lane it loads them as they lie (PER * 8 contiguous bytes per
    // lane); with many it loads tile j*64 + l, 512 contiguous bytes per instruction, and hands
    // each exp-sum to its owner through this wavefront's slice of LDS (rows of PER + 1 floats,
    // an odd stride, so both directions are conflict-free).
    constexpr bool EXCHANGE = PER > 10;
    __shared__ float exchange[EXCHANGE ? NW : 1][EXCHANGE ? kWave * (PER + 1) : 1];
    float2 p[PER];
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      const int t = EXCHANGE ? j * kWave + lane : lane * PER + j;
      p[j] = t < a.nT ? P[t] : make_float2(-INFINITY, 0.f);
      mx = fmaxf(mx, p[j].x);
    }
    mx = wave_max(mx);
#pragma unroll
    for (int j = 0; j < PER; ++j) mass[j] = p[j].y > 0.f ? p[j].y * expf(p[j].x - mx) : 0.f;
    if constexpr (EXCHANGE) {
      float* ex = exchange[wave];
#pragma unroll
      for (int j = 0; j < PER; ++j) {
        const int t = j * kWave + lane;
        ex[(t / PER) * (PER + 1) + t % PER] = mass[j];
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");  // same wavefront on both sides: order only
#pragma unroll
      for (int j = 0; j < PER; ++j) mass[j] = ex[lane * (PER + 1) + j];
    }
#pragma unroll
    for (int j = 0; j < PER; ++j) sm += mass[j];
  } else {
    for (int t = lane; t < a.nT; t += kWave) mx = fmaxf(mx, P[t].x);
    mx = wave_max(mx);
    for (int t = lane; t < a.nT; t += kWave) {
      const float2 p = P[t];
      sm += p.y * expf(p.x - mx);
    }
  }
  sm = wave_sum(sm);
  const float lse = mx + logf(sm);
  if (lane == 0) {
    a.lse[r] = lse;
    if (a.diag_lse) a.diag_lse[r] = lse;
  }
  if (!is_draft) {
    if (a.greedy) {  // point mass of the target law
      const int xt = row_argmax(a, P, a.logits + (size_t)r * a.ldl, mx);
      if (lane == 0) a.xtarget[s] = xt;
    }
    return;
  }

  int unresolved;
  const int pos = window_slot(a, b, m, unresolved);
  const int window = min(a.K, unresolved);
  if (lane == 0) {
    a.slot_pos[s] = pos;
    if (m == 0) a.window[b] = window;
  }
  int x = -1;
  if (m < window) {
    if (a.draft_tokens_in) {
      x = min(max(a.draft_tokens_in[s], 0), a.V - 1);  // keep the gathers in bounds
    } else if (a.greedy) {
      x = row_argmax(a, P, a.logits + (size_t)r * a.ldl, mx);  // point mass of the draft law
    } else {
      // x~ = min{v : sum_{w<=v} rho_w >= u}: first over vocabulary tiles, then inside the tile
      const float u = philox_uniform(a.seed, a.pos_base + (uint32_t)pos, a.step,
                                     a.seq_base + (uint32_t)b, kStreamDraft);
      Found tile;
      if constexpr (PER > 0) {
        const float inv = 1.f / sm;  // tile probability = exp-sum / row exp-sum
#pragma unroll
        for (int j = 0; j < PER; ++j) mass[j] *= inv;
        tile = wave_find_first_reg(mass, u);
      } else {
        tile = wave_find_first(
            a.nT, [&](int t) { const float2 p = P[t]; return p.y * expf(p.x - lse); }, u);
      }
      const float* L = a.logits + (size_t)r * a.ldl;
      const int v0 = tile_start(a, tile.idx);
      const int nv = min(tile_start(a, tile.idx + 1), a.V) - v0;
      Found in;
      if (nv <= kWave * kTilePer) {
        float q[kTilePer];
#pragma unroll
        for (int j = 0; j < kTilePer; ++j) {
          const int i = lane * kTilePer + j;
          q[j] = i < nv ? expf(L[v0 + i] - lse) : 0.f;
        }
        in = wave_find_first_reg(q, u - tile.before);
      } else {
        in = wave_find_first(nv, [&](int i) { return expf(L[v0 + i] - lse); }, u - tile.before);
      }
      x = v0 + in.idx;
    }
  }
  if (lane == 0) {
    a.xdraft[s] = x;
    if (a.diag_draft_tokens) a.diag_draft_tokens[s] = x;
    if (a.phase == 1) a.out_tokens[s] = x;  // draft-only call: the caller gets the draft tokens
  }
}

// ---------------------------------------------------------------------------------------------
// Final phase for one sequence (one workgroup): residual sample, commit, mask update, LowConf.
// ---------------------------------------------------------------------------------------------

// rm_pre: (wavefront 0 only) the residual chunk masses of this sequence, 16 per lane, loaded by the
// caller before the accept-phase results were known; valid if have_pre.
__device__ void finalize_sequence(const VerifyArgs& a, int b, const SeqState& st, BlockTmp& tmp,
                                  float* s_conf, uint8_t* s_mask, uint8_t* s_cand, const float (&rm_pre)[16],
                                  bool have_pre) {
  const int tid = threadIdx.x;
  const int BK = a.B * a.K;
  const int window = st.window, acc_len = st.acc_len;

  // diagnostics: overlap and residual mass of every slot
  if (a.all_slots) {
    for (int m = 0; m < a.K; ++m) {
      float al = 0.f, rm = 0.f;
      if (m < window) {
        const size_t base = (size_t)(b * a.K + m) * a.nRC;
        for (int c = tid; c < a.nRC; c += NT) {
          al += a.amass[base + c];
          rm += a.rmass[base + c];
        }
        al = block_sum(al, tmp);
        rm = block_sum(rm, tmp);
      }
      if (tid == 0) {
        if (a.diag_alpha) a.diag_alpha[b * a.K + m] = al;
        if (a.diag_resid_mass) a.diag_resid_mass[b * a.K + m] = rm;
      }
    }
  }

  // corrected token at the first rejection
  int z = -1;
  float z_conf = 0.f;
  if (acc_len < window) {
    const int s = b * a.K + acc_len;
    const float* Lq = a.logits + (size_t)s * a.ldl;
    const float* Lp = a.logits + (size_t)(BK + s) * a.ldl;
    // log-sum-exps, position and target arg max of the rejected slot travel with the accept-phase
    // results, so nothing here waits for a load whose address depends on acc_len except the logits
    const float lse_q = st.rej_lse_q, lse_p = st.rej_lse_p;
    const float* rm = a.rmass + (size_t)(a.all_slots ? s : b) * a.nRC;
    const float u = philox_uniform(a.seed, a.pos_base + (uint32_t)st.rej_pos, a.step,
                                   a.seq_base + (uint32_t)b, kStreamResidual);
    if (a.greedy) {
      z = st.rej_xtarget;  // residual of two point masses: the target's
      z_conf = expf(Lp[z] - lse_p);
    } else if (a.nRC <= kWave * kChunkPer) {
      // one wavefront, everything in registers
      if (tid < kWave) {
        float rmv[kChunkPer];
#pragma unroll
        for (int j = 0; j < kChunkPer; ++j) {
          const int c = tid * kChunkPer + j;
          rmv[j] = have_pre ? rm_pre[j] : (c < a.nRC ? rm[c] : 0.f);
        }
        const Found chunk = wave_find_first_reg<kChunkPer, true>(rmv, u);
        int zz;
        float zc;
        if (chunk.total > 0.f) {
          const int v0 = chunk.idx * kResidChunk + tid * 4;
          float qv[4] = {0.f, 0.f, 0.f, 0.f}, pv[4] = {0.f, 0.f, 0.f, 0.f};
          if (v0 + 3 < a.V) {
            const float4 q4 = *reinterpret_cast<const float4*>(Lq + v0);
            const float4 p4 = *reinterpret_cast<const float4*>(Lp + v0);
            qv[0] = q4.x; qv[1] = q4.y; qv[2] = q4.z; qv[3] = q4.w;
            pv[0] = p4.x; pv[1] = p4.y; pv[2] = p4.z; pv[3] = p4.w;
          } else {
            for (int j = 0; j < 4; ++j)
              if (v0 + j < a.V) { qv[j] = Lq[v0 + j]; pv[j] = Lp[v0 + j]; }
          }
          float rv[4], pe[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            pe[j] = expf(pv[j] - lse_p);
            rv[j] = v0 + j < a.V ? fmaxf(pe[j] - expf(qv[j] - lse_q), 0.f) : 0.f;
          }
          const Found in = wave_find_first_reg<4>(rv, u * chunk.total - chunk.before);
          zz = chunk.idx * kResidChunk + in.idx;
          // pi(z) from the lane that holds token z: no second trip to memory
          const int j = in.idx & 3;
          const float mine = j == 0 ? pe[0] : j == 1 ? pe[1] : j == 2 ? pe[2] : pe[3];
          zc = __shfl(mine, in.idx >> 2, 64);
        } else {
          // residual mass vanished in rounding although a rejection occurred: commit argmax pi
          float best = -INFINITY;
          int bi = INT_MAX;
          for (int v = tid; v < a.V; v += kWave) {
            const float l = Lp[v];
            if (l > best) { best = l; bi = v; }
          }
          const float gbest = wave_max(best);
          zz = wave_min_int(best == gbest ? bi : INT_MAX);
          zc = expf(Lp[zz] - lse_p);
        }
        if (tid == 0) { tmp.bcast_i = zz; tmp.bcast_f = zc; }
      }
      __syncthreads();
      z = tmp.bcast_i;
      z_conf = tmp.bcast_f;
    } else {
    float Z = 0.f;
    {
      const int per = (a.nRC + NT - 1) / NT;
      const int begin = min(a.nRC, tid * per), end = min(a.nRC, begin + per);
      float local = 0.f;
      for (int c = begin; c < end; ++c) local += rm[c];
      block_exclusive_scan(local, tmp, Z);
    }
    if (Z > 0.f) {
      const float target = u * Z;
      const Found chunk = block_find_first(a.nRC, [&](int c) { return rm[c]; }, target, tmp);
      const int v0 = chunk.idx * kResidChunk;
      const int nv = min(kResidChunk, a.V - v0);
      const Found in = block_find_first(
          nv,
          [&](int i) {
            return fmaxf(expf(Lp[v0 + i] - lse_p) - expf(Lq[v0 + i] - lse_q), 0.f);
          },
          target - chunk.before, tmp);
      z = v0 + in.idx;
    } else {
      // residual mass vanished in rounding although a rejection occurred: commit argmax pi
      float best = -INFINITY;
      int bi = INT_MAX;
      for (int v = tid; v < a.V; v += NT) {
        const float l = Lp[v];
        if (l > best) { best = l; bi = v; }
      }
      const float gbest = block_max(best, tmp);
      z = block_min_int(best == gbest ? bi : INT_MAX, tmp);
    }
    z_conf = expf(Lp[z] - lse_p);
    }
  }

  // commit tokens and confidences
  const int committed = min(acc_len + 1, window);
  if (tid < a.K) {
    const int s = b * a.K + tid;
    int tok = -1;
    float c = 0.f;
    if (tid < acc_len) { tok = st.x[tid]; c = st.ptok[tid]; }
    else if (tid == acc_len && acc_len < window) { tok = z; c = z_conf; }
    a.out_tokens[s] = tok;
    if (a.diag_conf_tok) a.diag_conf_tok[s] = c;
  }
  if (tid == 0) a.out_accept_len[b] = acc_len;

  // block state: mask, pass set, confidences
  const size_t row = (size_t)b * a.block;
  for (int i = tid; i < a.block; i += NT) {
    s_mask[i] = a.mask_in ? (a.mask_in[row + i] != 0) : 1;
    s_cand[i] = a.pass_mask ? (a.pass_mask[row + i] != 0) : 0;
    s_conf[i] = a.conf ? a.conf[row + i] : 0.f;
  }
  __syncthreads();
  if (tid < committed) {
    const int pos = a.slot_pos[b * a.K + tid];
    s_mask[pos] = 0;
    s_cand[pos] = 1;
    s_conf[pos] = (tid < acc_len) ? st.ptok[tid] : z_conf;
  }
  __syncthreads();
  int unresolved = 0;
  for (int i = tid; i < a.block; i += NT) unresolved |= s_mask[i];
  unresolved = block_max_int(unresolved, tmp);

  const bool final = a.seq_pass ? a.seq_pass[b] >= a.n_pass - 1 : a.final_pass != 0;
  const bool fire = !unresolved && !final;
  int remasked = 0;
  if (fire) {
    // LowConf: rank every candidate by (confidence, position); the n_rm lowest are re-masked
    const int n_rm = a.n_rm < 0 ? a.block / 2 : a.n_rm;
    for (int i = tid; i < a.block; i += NT) {
      const bool cand_i = a.lowconf_scope ? true : (s_cand[i] != 0);
      if (!cand_i) continue;
      const float ci = s_conf[i];
      int rank = 0;
      for (int j = 0; j < a.block; ++j) {
        const bool cand_j = a.lowconf_scope ? true : (s_cand[j] != 0);
        const float cj = s_conf[j];
        rank += (cand_j && (cj < ci || (cj == ci && j < i))) ? 1 : 0;
      }
      if (rank < n_rm) {
        // absorbing forward kernel: back to MASK with probability recorrupt_prob, else the
        // position keeps its token (both sides of u < prob are exact binary32 numbers)
        bool to_mask = true;
        if (a.recorrupt_prob < 1.f)
          to_mask = philox_uniform(a.seed, a.pos_base + (uint32_t)i, a.step, a.seq_base + (uint32_t)b,
                                   kStreamRecorrupt) < a.recorrupt_prob;
        if (to_mask) s_mask[i] = 1;
      }
    }
    __syncthreads();
    for (int i = tid; i < a.block; i += NT) remasked |= s_mask[i];
    remasked = block_max_int(remasked, tmp);
  }
  if (a.tokens_state && tid < committed)
    a.tokens_state[row + a.slot_pos[b * a.K + tid]] = tid < acc_len ? st.x[tid] : z;
  __syncthreads();  // seq_pass was read above by every thread; the token writes precede the -1s
  for (int i = tid; i < a.block; i += NT) {
    a.out_remask[row + i] = s_mask[i];
    if (a.pass_mask) a.pass_mask[row + i] = fire ? 0 : s_cand[i];
    if (a.conf) a.conf[row + i] = s_conf[i];
    if (a.tokens_state && fire && s_mask[i]) a.tokens_state[row + i] = -1;
  }
  if (tid == 0) {
    if (a.seq_pass) {
      if (fire && remasked) a.seq_pass[b] += 1;
      else if (!unresolved) a.seq_pass[b] = a.n_pass;  // final pass resolved, or nothing left to redo
    }
    if (a.seq_rounds && window > 0) a.seq_rounds[b] += 1;
  }
}

// ---------------------------------------------------------------------------------------------
// Kernel 2: accept tests, first rejection, residual / overlap mass per chunk.
// grid = (nslots, ceil(nRC / NW)); nslots = B (rejected slot only) or B*K (every slot).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(NT) void accept_resid_kernel(VerifyArgs a) {
  __shared__ SeqState st;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int BK = a.B * a.K;
  const int y = blockIdx.x;   // slot (all_slots) or sequence index
  const int cg = blockIdx.y;  // chunk group
  const int b = a.all_slots ? y / a.K : y;
  const int window = a.window[b];

  if (wave == 0) {
    // everything whose address is known up front is requested together (slots beyond the window
    // hold x = -1 and are not used); only the two gathers at x~ wait for a previous load
    const int sl = b * a.K + min(lane, a.K - 1);
    const int x = a.xdraft[sl], pos = a.slot_pos[sl];
    const float lse_q = a.lse[sl], lse_p = a.lse[BK + sl];
    const int xt = a.greedy ? a.xtarget[sl] : -1;
    bool rejected = false;
    if (lane < window) {
      const float lq = a.logits[(size_t)sl * a.ldl + x] - lse_q;
      const float lp = a.logits[(size_t)(BK + sl) * a.ldl + x] - lse_p;
      const float ratio = fminf(1.f, expf(lp - lq));
      const float u = philox_uniform(a.seed, a.pos_base + (uint32_t)pos, a.step,
                                     a.seq_base + (uint32_t)b, kStreamAccept);
      // greedy: the ratio of the two point masses is 1 if the arg maxes agree, else 0
      rejected = a.greedy ? x != xt : !(u <= ratio);
      st.x[lane] = x;
      st.ptok[lane] = expf(lp);
    }
    const unsigned long long rej = __ballot(rejected);
    const int acc = rej ? __ffsll((long long)rej) - 1 : window;
    if (lane == 0) {
      st.window = window;
      st.acc_len = acc;
    }
    if (lane == acc && acc < window) {  // the rejected slot's own values, for the final phase
      st.rej_lse_q = lse_q;
      st.rej_lse_p = lse_p;
      st.rej_pos = pos;
      st.rej_xtarget = xt;
    }
  }
  __syncthreads();
  if (cg == 0 && (!a.all_slots || y % a.K == 0) && tid < (int)(sizeof(SeqState) / 4))
    reinterpret_cast<int*>(a.seqstate + b)[tid] = reinterpret_cast<const int*>(&st)[tid];
  const int acc_len = st.acc_len;
  const int m = a.all_slots ? y % a.K : acc_len;
  const int c = cg * NW + wave;
  // chunk masses: not needed when nothing was rejected, for slots beyond the window, or in the
  // greedy variant (the corrected token is the target arg max) unless diagnostics want them
  if (m < window && c < a.nRC && (!a.greedy || a.all_slots)) {
    const int s = b * a.K + m;
    const float* Lq = a.logits + (size_t)s * a.ldl;
    const float* Lp = a.logits + (size_t)(BK + s) * a.ldl;
    const float lse_q = a.lse[s], lse_p = a.lse[BK + s];
    const int v = c * kResidChunk + lane * 4;
    float qv[4] = {0.f, 0.f, 0.f, 0.f}, pv[4] = {0.f, 0.f, 0.f, 0.f};
    if (v + 3 < a.V) {
      const float4 q4 = *reinterpret_cast<const float4*>(Lq + v);
      const float4 p4 = *reinterpret_cast<const float4*>(Lp + v);
      qv[0] = q4.x; qv[1] = q4.y; qv[2] = q4.z; qv[3] = q4.w;
      pv[0] = p4.x; pv[1] = p4.y; pv[2] = p4.z; pv[3] = p4.w;
    } else {
      for (int j = 0; j < 4; ++j)
        if (v + j < a.V) { qv[j] = Lq[v + j]; pv[j] = Lp[v + j]; }
    }
    float rs = 0.f, as = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (v + j < a.V) {
        const float q = expf(qv[j] - lse_q), p = expf(pv[j] - lse_p);
        rs += fmaxf(p - q, 0.f);
        as += fminf(p, q);
      }
    }
    rs = wave_sum(rs);
    if (a.all_slots) as = wave_sum(as);
    if (lane == 0) {
      a.rmass[(size_t)y * a.nRC + c] = rs;
      if (a.all_slots) a.amass[(size_t)y * a.nRC + c] = as;
    }
  }

}

// ---------------------------------------------------------------------------------------------
// Kernel 3: residual sample, commit, mask update, LowConf.  One workgroup per sequence.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(NT) void finalize_kernel(VerifyArgs a) {
  __shared__ BlockTmp tmp;
  __shared__ SeqState st;
  __shared__ float s_conf[kMaxBlock];
  __shared__ uint8_t s_mask[kMaxBlock], s_cand[kMaxBlock];
  const int b = blockIdx.x, tid = threadIdx.x;
  int word = 0;
  if (tid < (int)(sizeof(SeqState) / 4)) word = reinterpret_cast<const int*>(a.seqstate + b)[tid];
  // Without the diagnostics the chunk masses of a sequence sit at an address that does not depend
  // on which slot was rejected: wavefront 0 asks for them in the same breath as the accept-phase
  // results (when nothing was rejected they are stale and unused).
  float rm_pre[kChunkPer];
  const bool have_pre = !a.all_slots && !a.greedy && a.nRC <= kWave * kChunkPer;
#pragma unroll
  for (int j = 0; j < kChunkPer; ++j) {
    const int c = tid * kChunkPer + j;
    rm_pre[j] = (have_pre && tid < kWave && c < a.nRC) ? a.rmass[(size_t)b * a.nRC + c] : 0.f;
  }
  if (tid < (int)(sizeof(SeqState) / 4)) reinterpret_cast<int*>(&st)[tid] = word;
  __syncthreads();
  finalize_sequence(a, b, st, tmp, s_conf, s_mask, s_cand, rm_pre, have_pre);
}

// ---------------------------------------------------------------------------------------------
// Baseline step (parallel prediction with top-n confidence transfer): after kernel 1 has drawn a
// token for every window slot, one wavefront per sequence takes the confidences p(x) and commits
// the n most confident slots (equal confidences: the lower position first).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kWave) void topn_kernel(VerifyArgs a) {
  const int b = blockIdx.x, lane = threadIdx.x;
  const int window = a.window[b];
  const int s = b * a.K + lane;
  const bool live = lane < window;
  int x = -1, pos = INT_MAX;
  float c = -1.f;
  if (live) {
    x = a.xdraft[s];
    pos = a.slot_pos[s];
    c = expf(a.logits[(size_t)s * a.ldl + x] - a.lse[s]);
  }
  int rank = 0;
  for (int j = 0; j < window; ++j) {
    const float cj = __shfl(c, j, 64);
    const int pj = __shfl(pos, j, 64);
    rank += (cj > c || (cj == c && pj < pos)) ? 1 : 0;
  }
  const bool commit = live && rank < a.n_transfer;
  const size_t row = (size_t)b * a.block;
  if (lane < a.K) {
    a.out_tokens[s] = commit ? x : -1;
    if (a.diag_conf_tok) a.diag_conf_tok[s] = live ? c : 0.f;
  }
  if (lane == 0) a.out_accept_len[b] = min(a.n_transfer, window);
  for (int i = lane; i < a.block; i += kWave) a.out_remask[row + i] = a.mask_in ? (a.mask_in[row + i] != 0) : 1;
  __syncthreads();  // one wavefront: orders the mask copy before the committed positions are cleared
  if (commit) {
    a.out_remask[row + pos] = 0;
    if (a.conf) a.conf[row + pos] = c;
    if (a.tokens_state) a.tokens_state[row + pos] = x;
  }
}

__global__ void copy_logits_kernel(const float* __restrict__ src, long ldl, float* __restrict__ dst,
                                   int V, long rows) {
  const long n = rows * V;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < n; i += (long)gridDim.x * blockDim.x) {
    const long r = i / V, v = i - r * V;
    dst[i] = src[r * ldl + v];
  }
}

}  // namespace

hipError_t launch_verify(const VerifyArgs& a) {
  const dim3 g1((a.nrows + NW - 1) / NW);
  if (a.nT <= 64 * 4) hipLaunchKernelGGL(row_lse_draft_kernel<4>, g1, dim3(NT), 0, a.stream, a);
  else if (a.nT <= 64 * 8) hipLaunchKernelGGL(row_lse_draft_kernel<8>, g1, dim3(NT), 0, a.stream, a);
  else if (a.nT <= 64 * 10) hipLaunchKernelGGL(row_lse_draft_kernel<10>, g1, dim3(NT), 0, a.stream, a);  // 594 tiles of 256 tokens: V = 151936
  else if (a.nT <= 64 * 40) hipLaunchKernelGGL(row_lse_draft_kernel<40>, g1, dim3(NT), 0, a.stream, a);
  else hipLaunchKernelGGL(row_lse_draft_kernel<0>, g1, dim3(NT), 0, a.stream, a);
  if (a.phase == 3) {
    hipLaunchKernelGGL(topn_kernel, dim3(a.B), dim3(kWave), 0, a.stream, a);
  } else if (a.phase != 1) {  // everything after the draft sample needs the target laws
    const int gx = (a.nRC + NW - 1) / NW;
    const int nslots = a.all_slots ? a.B * a.K : a.B;
    hipLaunchKernelGGL(accept_resid_kernel, dim3(nslots, gx), dim3(NT), 0, a.stream, a);
    hipLaunchKernelGGL(finalize_kernel, dim3(a.B), dim3(NT), 0, a.stream, a);
  }
  if (a.diag_logits) {
    const long rows = a.nrows;
    const long n = rows * a.V;
    const int blocks = (int)((n + 255) / 256 > 65535 ? 65535 : (n + 255) / 256);
    hipLaunchKernelGGL(copy_logits_kernel, dim3(blocks), dim3(256), 0, a.stream,
                       a.logits + (size_t)a.row0 * a.ldl, a.ldl, a.diag_logits + (size_t)a.row0 * a.V, a.V, rows);
  }
  return hipGetLastError();
}

}  // namespace fef
