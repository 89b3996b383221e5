// Vocabulary-head kernels: L[r, v] = inv_tau * sum_k H[r, k] W[v, k] for the draft rows
// followed by the target rows (the two laws of Algorithm 2, "Compute draft laws" and "Compute
// target laws", share one pass over W because the paper uses one network for both), fp32
// logits written once, and per (row, vocabulary tile) partials (max, sum exp(L - max)) from
// which the row's log-sum-exp is merged later.
//
//   head_skinny_kernel  M = 2*B*K <= 16 (head_skinny32_kernel: 16 < M <= 32, see there).
//                       HBM-bound: W (about 1 GB) is streamed exactly once.
//                       One workgroup per CU owns a contiguous run of 16-token tiles.  Its
//                       eight wavefronts split k; each keeps its slice of H in registers as
//                       the MFMA B operand for the whole kernel, streams its 1 KB slice of
//                       sixteen W rows straight into the MFMA A operand registers one tile
//                       ahead, and the eight partial 16x16 tiles are summed through LDS.
//                       One (max, sum exp) partial per (row, workgroup).
//   head_tiled_kernel   any M.  128x128x64 LDS-tiled MFMA GEMM, XCD-aware tile order so the
//                       workgroups that share a W tile run on the same L2.
//   head_f32_kernel     fp32 inputs, plain FMA; tiny instances only.
#include <type_traits>

#include "head_common.hpp"

namespace fef {
namespace {

// ---------------------------------------------------------------------------------------------
// Skinny kernel.  KS = MFMA k-steps (32 wide) per wavefront; d = 8 * KS * 32.
//
// v_mfma_f32_16x16x32_bf16 operand layout (lane l, i = l % 16, g = l / 16):
//   A (16 x 32): lane holds A[i][8g .. 8g+7]        -> W tile row i, 16 contiguous bytes
//   B (32 x 16): lane holds B[8g .. 8g+7][i]        -> H row i, the same k range
//   D (16 x 16): lane holds D[4g + r][i], r = 0..3  -> logits of 4 consecutive tokens, row i
// ---------------------------------------------------------------------------------------------
#ifndef FEF_NT_LOGITS
#define FEF_NT_LOGITS 1
#endif
// The logits of a workgroup leave in one burst at its end, i.e. all 8 to 16 MB of them in the last
// microseconds of the kernel.  Written as ordinary stores they would sit dirty in L2 until the
// write-back that closes the kernel, which the next kernel has to wait for; non-temporal stores
// go through to memory at once.
__device__ inline void store_logit(float* p, float v) {
#if FEF_NT_LOGITS
  __builtin_nontemporal_store(v, p);
#else
  *p = v;
#endif
}

constexpr int kSkinnyWaves = 8;
constexpr int kSkinnyOutTiles = 40;  // tiles of logits staged in LDS before a flush
constexpr int kSkinnyThreads = kSkinnyWaves * kWave;

// NB = tiles accumulated in registers between two cross-wavefront reductions (even).
template <int KS, int NB>
__global__ __launch_bounds__(kSkinnyThreads) void head_skinny_kernel(HeadArgs a, int tiles_total) {
  static_assert(NB * 64 <= kSkinnyThreads, "one reduction item per thread at most");
  __shared__ floatx4 red[2][NB][kSkinnyWaves][kWave];
  __shared__ float2 run_merge[NB][16];
  // Logits of this workgroup's tokens wait here and leave in one coalesced burst: a global
  // store inside the streaming loop would share the vector-memory counter with the W
  // prefetch and force every wait on a W tile to drain the tiles fetched ahead as well.
  __shared__ __attribute__((aligned(16))) float out[16][kSkinnyOutTiles * 16 + 16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i16 = lane & 15, g = lane >> 4;
  const int M = a.nrows;
  const int kofs = wave * (KS * 32) + g * 8;  // first k of this lane; k-step s adds 32 s

  bf16x8 hreg[KS];
  {
    const bool live = i16 < M;
    const __bf16* hp = h_row(a, live ? i16 : 0) + kofs;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      bf16x8 v = *reinterpret_cast<const bf16x8*>(hp + 32 * s);
      if (!live) v = bf16x8{};
      hreg[s] = v;
    }
  }

  const int t0 = (int)((long)blockIdx.x * tiles_total / gridDim.x);
  const int t1 = (int)((long)(blockIdx.x + 1) * tiles_total / gridDim.x);
  const __bf16* Wl = (const __bf16*)a.W + kofs;

  auto load_tile = [&](int t, bf16x8(&buf)[KS]) {
    const int v = min(t * 16 + i16, a.V - 1);  // rows past V re-read the last row, masked later
    const __bf16* wp = Wl + (size_t)v * a.d;
#pragma unroll
    for (int s = 0; s < KS; ++s) buf[s] = *reinterpret_cast<const bf16x8*>(wp + 32 * s);
  };
  auto mfma_tile = [&](const bf16x8(&buf)[KS]) {
    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < KS; ++s)
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(buf[s], hreg[s], acc, 0, 0, 0);
    return acc;
  };

  // Reduction item of this thread inside a batch (threads 0..64 NB - 1): tile jt_o of the
  // batch, row m, tokens 4 quad .. 4 quad + 3.  The D layout puts exactly those four sums in
  // lane m + 16 quad of every wavefront's accumulator.
  const int jt_o = tid >> 6, m = (tid >> 2) & 15, quad = tid & 3;
  const int src = m + 16 * quad;
  // running (max, sum exp) over this thread's tiles, replicated over the item's 4 lanes
  float run_m = -INFINITY, run_s = 0.f;

  // W prefetch.  The order and grouping of a wavefront's loads decide the rate of the whole kernel;
  // what follows was found with a read-only kernel of this access pattern and confirmed here.
  // (1) Loads go out in bursts of about 8 (of 1 KB each): a read-only kernel gets 6.4 to 6.6 TB/s with
  // bursts of 8, 6.2 with 4 and 5.9 with 16, and one load after each multiply is slower than any of
  // these.  So a tile of 10 or more k-steps is fetched as two halves, each requested again as soon
  // as it has been multiplied; shorter tiles are fetched whole, one tile ahead, into two buffers.
  // (2) Inside a burst the LAST 64-byte piece of the half goes first, then the others in ascending
  // order: 4 to 5 % faster than ascending order throughout (165 against 169 us at d = 4096, V =
  // 126464); any order that touches both 256-byte blocks of the half within its first two loads
  // does as well, strictly alternating ones do not.
  // (3) No tile is fetched or multiplied twice to make the loop uniform: one extra tile per workgroup
  // (a thirtieth of its work) costs its full time although it hits in cache.
  constexpr bool kHalves = KS >= 10;
  constexpr int GA = kHalves ? KS / 2 : KS, GB = kHalves ? KS - GA : KS;
  bf16x8 buf0[GA], buf1[GB];
  auto load_half = [&](int t, auto half, auto& buf) {
    constexpr int H = decltype(half)::value;
    constexpr int G = H ? GB : GA;
    const int v = min(t * 16 + i16, a.V - 1);
    const __bf16* wp = Wl + (size_t)v * a.d + 32 * (H * GA);
    buf[G - 1] = *reinterpret_cast<const bf16x8*>(wp + 32 * (G - 1));
    asm volatile("" ::: "memory");  // keeps the order of the requests
#pragma unroll
    for (int s = 0; s < G - 1; ++s) {
      buf[s] = *reinterpret_cast<const bf16x8*>(wp + 32 * s);
      asm volatile("" ::: "memory");
    }
  };
  using Half0 = std::integral_constant<int, 0>;
  using Half1 = std::integral_constant<int, 1>;
  floatx4 acc[NB];
  int par = 0;
  int tflush = t0;  // first tile whose logits are still staged in LDS
  if (t0 < t1) {
    if constexpr (kHalves) {
      load_half(t0, Half0{}, buf0);
      load_half(t0, Half1{}, buf1);
    } else {
      load_tile(t0, buf0);
    }
  }
  for (int t = t0; t < t1; t += NB) {
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      if (t + i < t1) {
        if constexpr (kHalves) {
          floatx4 c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int s = 0; s < GA; ++s) c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(buf0[s], hreg[s], c, 0, 0, 0);
          if (t + i + 1 < t1) load_half(t + i + 1, Half0{}, buf0);
#pragma unroll
          for (int s = 0; s < GB; ++s) c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(buf1[s], hreg[GA + s], c, 0, 0, 0);
          if (t + i + 1 < t1) load_half(t + i + 1, Half1{}, buf1);
          acc[i] = c;
        } else if (i & 1) {
          if (t + i + 1 < t1) load_tile(t + i + 1, buf0);
          acc[i] = mfma_tile(buf1);
        } else {
          if (t + i + 1 < t1) load_tile(t + i + 1, buf1);
          acc[i] = mfma_tile(buf0);
        }
      }
    }
    const int nb = min(NB, t1 - t);
#pragma unroll
    for (int i = 0; i < NB; ++i)
      if (i < nb) red[par][i][wave][lane] = acc[i];
    lds_barrier();
    // sum the eight k-slices in wave order
    if (jt_o < nb) {
      floatx4 sum = red[par][jt_o][0][src];
#pragma unroll
      for (int w = 1; w < kSkinnyWaves; ++w) sum += red[par][jt_o][w][src];
      sum *= a.inv_tau;
      const int v = (t + jt_o) * 16 + 4 * quad;
      *reinterpret_cast<floatx4*>(&out[m][(t + jt_o - tflush) * 16 + 4 * quad]) = sum;
      float mx = -INFINITY;
#pragma unroll
      for (int c = 0; c < 4; ++c)
        if (v + c < a.V && m < M) mx = fmaxf(mx, sum[c]);
      mx = fmaxf(mx, __shfl_xor(mx, 1, 64));
      mx = fmaxf(mx, __shfl_xor(mx, 2, 64));
      float e = 0.f;
#pragma unroll
      for (int c = 0; c < 4; ++c)
        if (v + c < a.V && m < M) e += __expf(sum[c] - mx);
      e += __shfl_xor(e, 1, 64);
      e += __shfl_xor(e, 2, 64);
      if (mx > run_m) { run_s = run_s * __expf(run_m - mx) + e; run_m = mx; }
      else if (mx > -INFINITY) run_s += e * __expf(mx - run_m);
    }
    par ^= 1;
    if (t + NB - tflush + NB > kSkinnyOutTiles || t + NB >= t1) {
      // flush rows [tflush*16, min(t+NB, t1)*16) of the staged logits
      const int tend = min(t + NB, t1);
      const int v0 = tflush * 16, nv = min(tend * 16, a.V) - v0;
      __syncthreads();
      for (int r = wave; r < M; r += kSkinnyWaves)
        for (int i = lane; i < nv; i += kWave) store_logit(&a.logits[(size_t)r * a.ldl + v0 + i], out[r][i]);
      __syncthreads();
      tflush = tend;
    }
  }

  // merge the NB items that share a row and write the workgroup's partial
  if (quad == 0 && jt_o < NB) run_merge[jt_o][m] = make_float2(run_m, run_s);
  __syncthreads();
  if (tid < 16 && tid < M) {
    float mx = -INFINITY;
#pragma unroll
    for (int j = 0; j < NB; ++j) mx = fmaxf(mx, run_merge[j][tid].x);
    float sm = 0.f;
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const float2 pj = run_merge[j][tid];
      if (pj.x > -INFINITY) sm += pj.y * __expf(pj.x - mx);
    }
    a.partials[(size_t)tid * a.nT + blockIdx.x] = make_float2(mx, sm);
  }
}

// ---------------------------------------------------------------------------------------------
// Skinny kernel for 16 < M <= 32 (a 16-token window at B = 1, or two 8-token windows): the same
// streaming scheme with two 16-row groups of H resident per wavefront (2 * KS operand
// registers), each W tile multiplied against both.  The register budget then leaves room for
// one W buffer only: the next tile's loads are issued right after the multiplies that consumed
// the current one, which keeps one 16 KB tile per wavefront (128 KB per CU) in flight.
// The reduction buffer is single (two barriers per batch) so that it and the 32-row logits
// staging fit in LDS together.
// ---------------------------------------------------------------------------------------------
template <int KS, int NB>
__global__ __launch_bounds__(kSkinnyThreads) void head_skinny32_kernel(HeadArgs a, int tiles_total) {
  static_assert(NB * 128 == kSkinnyThreads, "one reduction item per thread");
  __shared__ floatx4 red[NB][2][kSkinnyWaves][kWave];
  __shared__ float2 run_merge[NB][32];
  __shared__ __attribute__((aligned(16))) float out[32][kSkinnyOutTiles * 16 + 16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i16 = lane & 15, g = lane >> 4;
  const int M = a.nrows;
  const int kofs = wave * (KS * 32) + g * 8;

  bf16x8 hreg[2][KS];
#pragma unroll
  for (int mt = 0; mt < 2; ++mt) {
    const int r = mt * 16 + i16;
    const bool live = r < M;
    const __bf16* hp = h_row(a, live ? r : 0) + kofs;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      bf16x8 v = *reinterpret_cast<const bf16x8*>(hp + 32 * s);
      if (!live) v = bf16x8{};
      hreg[mt][s] = v;
    }
  }

  const int t0 = (int)((long)blockIdx.x * tiles_total / gridDim.x);
  const int t1 = (int)((long)(blockIdx.x + 1) * tiles_total / gridDim.x);
  const __bf16* Wl = (const __bf16*)a.W + kofs;

  // One W buffer of KS registers, refilled in two halves (tiles of 10 or more k-steps): a half is
  // requested again, as one burst with its last piece first, as soon as its multiplies are done
  // (see the kernel for M <= 16 for what the grouping and the order are worth).
  constexpr bool kHalves = KS >= 10;
  constexpr int GA = kHalves ? KS / 2 : KS;
  bf16x8 buf[KS];
  auto load_part = [&](int t, int s0, int s1) {
    const int v = min(t * 16 + i16, a.V - 1);
    const __bf16* wp = Wl + (size_t)v * a.d;
    if (kHalves) {  // a burst: its last piece first
      buf[s1 - 1] = *reinterpret_cast<const bf16x8*>(wp + 32 * (s1 - 1));
      asm volatile("" ::: "memory");
    }
#pragma unroll
    for (int s = s0; s < s1 - (kHalves ? 1 : 0); ++s) {
      buf[s] = *reinterpret_cast<const bf16x8*>(wp + 32 * s);
      asm volatile("" ::: "memory");
    }
  };

  // Reduction item of this thread inside a batch: tile jt_o, row group mt_o, row m of it,
  // tokens 4 quad .. 4 quad + 3 (64 NB * 2 items; NB = 4 gives every thread one).
  const int jt_o = tid >> 7, mt_o = (tid >> 6) & 1, m = (tid >> 2) & 15, quad = tid & 3;
  const int row = mt_o * 16 + m;
  const int src = m + 16 * quad;
  float run_m = -INFINITY, run_s = 0.f;

  floatx4 acc[NB][2];
  int tflush = t0;
  if (t0 < t1) load_part(t0, 0, KS);
  for (int t = t0; t < t1; t += NB) {
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      if (t + i < t1) {
        floatx4 c0 = {0.f, 0.f, 0.f, 0.f}, c1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < GA; ++s) {
          c0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(buf[s], hreg[0][s], c0, 0, 0, 0);
          c1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(buf[s], hreg[1][s], c1, 0, 0, 0);
        }
        if (t + i + 1 < t1) load_part(t + i + 1, 0, GA);
        if constexpr (kHalves) {
#pragma unroll
          for (int s = GA; s < KS; ++s) {
            c0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(buf[s], hreg[0][s], c0, 0, 0, 0);
            c1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(buf[s], hreg[1][s], c1, 0, 0, 0);
          }
          if (t + i + 1 < t1) load_part(t + i + 1, GA, KS);
        }
        acc[i][0] = c0;
        acc[i][1] = c1;
      }
    }
    const int nb = min(NB, t1 - t);
    lds_barrier();  // every thread has finished reading the previous batch
#pragma unroll
    for (int i = 0; i < NB; ++i)
      if (i < nb) {
        red[i][0][wave][lane] = acc[i][0];
        red[i][1][wave][lane] = acc[i][1];
      }
    lds_barrier();
    if (jt_o < nb) {
      floatx4 sum = red[jt_o][mt_o][0][src];
#pragma unroll
      for (int w = 1; w < kSkinnyWaves; ++w) sum += red[jt_o][mt_o][w][src];
      sum *= a.inv_tau;
      const int v = (t + jt_o) * 16 + 4 * quad;
      *reinterpret_cast<floatx4*>(&out[row][(t + jt_o - tflush) * 16 + 4 * quad]) = sum;
      float mx = -INFINITY;
#pragma unroll
      for (int c = 0; c < 4; ++c)
        if (v + c < a.V && row < M) mx = fmaxf(mx, sum[c]);
      mx = fmaxf(mx, __shfl_xor(mx, 1, 64));
      mx = fmaxf(mx, __shfl_xor(mx, 2, 64));
      float e = 0.f;
#pragma unroll
      for (int c = 0; c < 4; ++c)
        if (v + c < a.V && row < M) e += __expf(sum[c] - mx);
      e += __shfl_xor(e, 1, 64);
      e += __shfl_xor(e, 2, 64);
      if (mx > run_m) { run_s = run_s * __expf(run_m - mx) + e; run_m = mx; }
      else if (mx > -INFINITY) run_s += e * __expf(mx - run_m);
    }
    if (t + NB - tflush + NB > kSkinnyOutTiles || t + NB >= t1) {
      const int tend = min(t + NB, t1);
      const int v0 = tflush * 16, nv = min(tend * 16, a.V) - v0;
      __syncthreads();
      for (int r = wave; r < M; r += kSkinnyWaves)
        for (int i = lane; i < nv; i += kWave) store_logit(&a.logits[(size_t)r * a.ldl + v0 + i], out[r][i]);
      __syncthreads();
      tflush = tend;
    }
  }
  // merge the NB items that share a row and write the workgroup's partial
  if (quad == 0) run_merge[jt_o][row] = make_float2(run_m, run_s);
  __syncthreads();
  if (tid < 32 && tid < M) {
    float mx = -INFINITY;
#pragma unroll
    for (int j = 0; j < NB; ++j) mx = fmaxf(mx, run_merge[j][tid].x);
    float sm = 0.f;
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const float2 pj = run_merge[j][tid];
      if (pj.x > -INFINITY) sm += pj.y * __expf(pj.x - mx);
    }
    a.partials[(size_t)tid * a.nT + blockIdx.x] = make_float2(mx, sm);
  }
}

// ---------------------------------------------------------------------------------------------
// Tiled kernel: workgroup tile 128 (rows of H) x 128 (tokens) x 64 (k), four wavefronts in a
// 2 x 2 grid, each 64 x 64 as 2 x 2 v_mfma_f32_32x32x16_bf16 tiles.
//
// 32x32x16 operand layout (lane l, j = l % 32, h = l / 32):
//   A (32 x 16): lane holds A[j][8h .. 8h+7]     -> H row j
//   B (16 x 32): lane holds B[8h .. 8h+7][j]     -> W row (token) j
//   D (32 x 32): lane holds D[8 (r/4) + 4h + r%4][j], r = 0..15
// LDS tiles are [128 rows][64 k] bf16 = 128 B per row; the eight 16-byte chunks of a row are
// stored at chunk ^ (row & 7) so the 16-byte reads of one k-chunk over 32 rows spread over all
// banks.
// ---------------------------------------------------------------------------------------------
constexpr int TM = 128, TN = 128, TK = 64;
constexpr int kTiledThreads = 256;

__global__ __launch_bounds__(kTiledThreads) void head_tiled_kernel(HeadArgs a, int m_tiles, int n_tiles) {
  __shared__ bf16x8 As[TM * 8];
  __shared__ bf16x8 Bs[TN * 8];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int j32 = lane & 31, h = lane >> 5;
  const int M = a.nrows;

  // XCD-aware order: workgroup ids round-robin over the 8 XCDs, so ids with the same id % 8
  // share an L2.  Within one XCD, consecutive workgroups walk the row tiles of one token tile.
  const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
  const int nt = xcd + 8 * (seq / m_tiles), mt = seq % m_tiles;
  if (nt >= n_tiles) return;
  const int m0 = mt * TM, n0 = nt * TN;

  // global -> register staging: thread loads chunk (tid % 8) of rows tid/8 + 32 j, j = 0..3
  const int lc = tid & 7, lr = tid >> 3;
  const __bf16* ap[4];
  const __bf16* bp[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int r = min(m0 + lr + 32 * j, M - 1);
    const int v = min(n0 + lr + 32 * j, a.V - 1);
    ap[j] = h_row(a, r) + lc * 8;
    bp[j] = (const __bf16*)a.W + (size_t)v * a.d + lc * 8;
  }
  bf16x8 ra[4], rb[4];
  auto gload = [&](int k0) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      ra[j] = *reinterpret_cast<const bf16x8*>(ap[j] + k0);
      rb[j] = *reinterpret_cast<const bf16x8*>(bp[j] + k0);
    }
  };

  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = floatx16{};

  gload(0);
  for (int k0 = 0; k0 < a.d; k0 += TK) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      As[swz(lr + 32 * j, lc)] = ra[j];
      Bs[swz(lr + 32 * j, lc)] = rb[j];
    }
    lds_barrier();
    if (k0 + TK < a.d) gload(k0 + TK);
#pragma unroll
    for (int ks = 0; ks < TK / 16; ++ks) {
      bf16x8 af[2], bf[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        af[i] = As[swz(wm * 64 + i * 32 + j32, ks * 2 + h)];
        bf[i] = Bs[swz(wn * 64 + i * 32 + j32, ks * 2 + h)];
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
    }
    lds_barrier();
  }

  // epilogue: scale, store, per-row (max, sum exp) over this wavefront's 64 tokens
  const int vbase = n0 + wn * 64;
  const int ptile = vbase / kTiledTn;
  const bool tile_live = vbase < a.V;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = m0 + wm * 64 + i * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
      const int v0 = vbase + j32, v1 = v0 + 32;
      const float l0 = acc[i][0][r] * a.inv_tau, l1 = acc[i][1][r] * a.inv_tau;
      const bool ok0 = m < M && v0 < a.V, ok1 = m < M && v1 < a.V;
      if (ok0) a.logits[(size_t)m * a.ldl + v0] = l0;
      if (ok1) a.logits[(size_t)m * a.ldl + v1] = l1;
      float mx = fmaxf(ok0 ? l0 : -INFINITY, ok1 ? l1 : -INFINITY);
#pragma unroll
      for (int off = 16; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
      float e = (ok0 ? __expf(l0 - mx) : 0.f) + (ok1 ? __expf(l1 - mx) : 0.f);
#pragma unroll
      for (int off = 16; off >= 1; off >>= 1) e += __shfl_xor(e, off, 64);
      if (j32 == 0 && m < M && tile_live) a.partials[(size_t)m * a.nT + ptile] = make_float2(mx, e);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// fp32 kernel: one wavefront per (row, 64-token tile), lane = token, sequential FMA over k.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kWave) void head_f32_kernel(HeadArgs a) {
  const int lane = threadIdx.x;
  const int t = blockIdx.x, r = blockIdx.y;
  const int v = t * kTiledTn + lane;
  const bool valid = v < a.V;
  const int g = a.row0 + r;
  const float* hp = g < a.BK ? (const float*)a.h_draft + (size_t)g * a.d
                             : (const float*)a.h_target + (size_t)(g - a.BK) * a.d;
  const float* wp = (const float*)a.W + (size_t)(valid ? v : a.V - 1) * a.d;
  float acc = 0.f;
  for (int k = 0; k < a.d; ++k) acc = fmaf(hp[k], wp[k], acc);
  const float logit = acc * a.inv_tau;
  if (a.labels) {  // cross-entropy use: keep only the label token's logit
    if (valid && a.labels[r] == v) a.label_logit[r] = logit;
  } else if (valid) {
    a.logits[(size_t)r * a.ldl + v] = logit;
  }
  float mx = valid ? logit : -INFINITY;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
  float e = valid ? expf(logit - mx) : 0.f;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) e += __shfl_xor(e, off, 64);
  if (lane == 0) a.partials[(size_t)r * a.nT + t] = make_float2(mx, e);
}

}  // namespace

// The eight wavefronts split k into slices of 32 KS columns held in registers: d = 256 KS with KS
// fixed at compile time; instantiated for the hidden sizes below.
#define FEF_SKINNY_SIZES(X) X(512, 2) X(1024, 4) X(2048, 8) X(2560, 10) X(3072, 12) X(3584, 14) X(4096, 16)

bool skinny_supports(int M, int d) {
  if (M > 32) return false;
#define FEF_X(D, KS) if (d == D) return true;
  FEF_SKINNY_SIZES(FEF_X)
#undef FEF_X
  return false;
}

template <int NB>
hipError_t launch_head_skinny_nb(const HeadArgs& a) {
  const int tiles = (a.V + kSkinnyUnit - 1) / kSkinnyUnit;
  const int grid = a.nT;  // = min(tiles, kSkinnyMaxGrid): one partial per (row, workgroup)
  switch (a.d) {
#define FEF_X(D, KS)                                                                                         \
  case D:                                                                                                    \
    if (a.nrows > 16)                                                                                        \
      FEF_LAUNCH_HEAD((head_skinny32_kernel<KS, NB>), dim3(grid), dim3(kSkinnyThreads), a, a, tiles);        \
    else                                                                                                     \
      FEF_LAUNCH_HEAD((head_skinny_kernel<KS, NB>), dim3(grid), dim3(kSkinnyThreads), a, a, tiles);          \
    break;
    FEF_SKINNY_SIZES(FEF_X)
#undef FEF_X
    default:
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_head_skinny(const HeadArgs& a) { return launch_head_skinny_nb<4>(a); }

hipError_t launch_head_tiled(const HeadArgs& a) {
  const int M = a.nrows;
  const int m_tiles = (M + TM - 1) / TM, n_tiles = (a.V + TN - 1) / TN;
  const long grid = 8L * ((n_tiles + 7) / 8) * m_tiles;
  FEF_LAUNCH_HEAD(head_tiled_kernel, dim3((unsigned)grid), dim3(kTiledThreads), a, a, m_tiles, n_tiles);
  return hipGetLastError();
}

hipError_t launch_head_f32(const HeadArgs& a) {
  FEF_LAUNCH_HEAD(head_f32_kernel, dim3(a.nT, a.nrows), dim3(kWave), a, a);
  return hipGetLastError();
}

}  // namespace fef
