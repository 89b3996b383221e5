// Vocabulary-head kernel for large M = 2*B*K (the batched, MFMA-bound configurations).
//
// Workgroup tile 256 (rows of H) x 256 (tokens), k-steps of 32; eight wavefronts in a 2 x 4 grid,
// each 128 x 64 as 4 x 2 v_mfma_f32_32x32x16_bf16 tiles (128 accumulator registers).
//
// Operand slabs go HBM/L2 -> LDS directly (global_load_lds_dwordx4: lane l of a wavefront
// deposits its 16 bytes at LDS base + 16 l, so one instruction fills 1 KB = 16 rows x 64 B) into
// a ring of four 32 KB stages, issued three k-steps ahead of their use; no register staging and
// no ds_write in the main loop.  A stage is [256 rows][4 chunks of 16 B] for A and for B.  The
// LDS has 64 four-byte banks, i.e. four 64-byte rows per sweep, so chunk c of row r is kept at
// position c ^ ((r >> 2) & 3): the 16-byte fragment reads of 16 consecutive rows then touch
// every bank once.  The permutation is applied on the global side (each lane fetches the chunk
// that belongs in its LDS slot).
//
// The epilogue works straight from the accumulator registers: for a fixed accumulator index the 32
// lanes of a half-wavefront hold 32 consecutive tokens of one row, so dword stores write whole
// 128-byte lines, and the per-row (max, sum exp) over the wavefront's 64 tokens is reduced by DPP.
//
// Tile order: workgroup ids go round-robin over the 8 XCDs; within an XCD consecutive
// workgroups take the row tiles of one token tile, so a W tile comes from HBM once and is
// shared through that XCD's L2.
#include "head_common.hpp"

namespace fef {
namespace {

constexpr int BM = 256, BN = 256, BK = 32;
constexpr int kStageChunks = (BM + BN) * 4;  // 16-byte chunks per stage: A rows then B rows

__device__ inline int swz4(int row, int chunk) { return row * 4 + (chunk ^ ((row >> 2) & 3)); }

// global_load_lds_dwordx4: lane l copies 16 bytes from its global address to LDS offset
// lds_off + 16 l (lds_off wavefront-uniform, carried in M0).  Written as inline assembly so
// that the compiler's wait-count pass does not tie the fragment reads of one stage to the
// loads still in flight for the others (it would drain them all once per ring cycle);
// completion is tracked by hand with vmcnt before the workgroup barrier.
__device__ inline void load_to_lds_16(const void* gptr, uint32_t lds_off) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :: "v"(gptr), "s"(lds_off) : "memory");
}
// Wait until at most N of this wavefront's vector-memory operations are outstanding.
template <int N>
__device__ inline void wait_newer() {
  static_assert(N == 0 || N == 4 || N == 8 || N == 16, "add the count");
  if constexpr (N == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  if constexpr (N == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
  if constexpr (N == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
  if constexpr (N == 16) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
}
// max(x, x rotated right by N inside its row of 16 lanes) in one instruction.  The s_nop covers
// the two wait states a DPP read needs after a vector write of its source.
template <int N>
__device__ inline float max_ror(float x) {
  static_assert(N == 1 || N == 2 || N == 4 || N == 8, "add the rotation");
  float r;
  if constexpr (N == 8) asm("s_nop 1\n\tv_max_f32_dpp %0, %1, %1 row_ror:8 row_mask:0xf bank_mask:0xf" : "=v"(r) : "v"(x));
  if constexpr (N == 4) asm("s_nop 1\n\tv_max_f32_dpp %0, %1, %1 row_ror:4 row_mask:0xf bank_mask:0xf" : "=v"(r) : "v"(x));
  if constexpr (N == 2) asm("s_nop 1\n\tv_max_f32_dpp %0, %1, %1 row_ror:2 row_mask:0xf bank_mask:0xf" : "=v"(r) : "v"(x));
  if constexpr (N == 1) asm("s_nop 1\n\tv_max_f32_dpp %0, %1, %1 row_ror:1 row_mask:0xf bank_mask:0xf" : "=v"(r) : "v"(x));
  return r;
}
__device__ inline uint32_t lds_offset(const void* p) {
  return __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)p);
}

// TJ = 32-token tiles per wavefront: 2 -> eight wavefronts of 128 x 64 (used), 4 -> four of
// 128 x 128 (one wavefront per SIMD; measured slower: 874 vs 920 TFLOP/s at M = 2048).
template <int TJ>
__global__ __launch_bounds__(2 * (BN / (32 * TJ)) * kWave) void head_tiled256_kernel(HeadArgs a, int m_tiles, int n_tiles) {
  constexpr int WN = BN / (32 * TJ);      // wavefronts along the token dimension
  constexpr int NWAVES = 2 * WN;
  constexpr int QI = BM / (16 * NWAVES);  // load instructions per operand per wavefront per stage
  // one array per stage, so the compiler can tell the in-flight LDS writes of the other stages
  // from the fragment reads of the current one
  __shared__ bf16x8 st0[kStageChunks], st1[kStageChunks], st2[kStageChunks], st3[kStageChunks];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: LDS offsets of the loads need no lane readback
  const int wm = wave / WN, wn = wave % WN;
  const int j32 = lane & 31, h = lane >> 5;
  const int M = a.nrows;

  const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
  const int nt = xcd + 8 * (seq / m_tiles), mt = seq % m_tiles;
  if (nt >= n_tiles) return;
  const int m0 = mt * BM, n0 = nt * BN;

  // Direct-to-LDS loads: wavefront w fills rows [32 w, 32 w + 32) of A and of B, 16 rows per
  // instruction; lane l owns LDS slot (row 16 q + l/4, position l%4) and fetches the chunk that
  // the swizzle assigns to that slot.
  const __bf16* gp[2 * QI];
#pragma unroll
  for (int q = 0; q < QI; ++q) {
    const int rl = wave * (16 * QI) + q * 16 + (lane >> 2);  // row inside the tile
    const int c = (lane & 3) ^ ((rl >> 2) & 3);            // logical 16-byte chunk of that row
    const int r = min(m0 + rl, M - 1);                     // rows past M / V re-read the last
    const int v = min(n0 + rl, a.V - 1);                   // row; masked in the epilogue
    gp[q] = h_row(a, r) + c * 8;
    gp[QI + q] = (const __bf16*)a.W + (size_t)v * a.d + c * 8;
  }
  // gp[] point at k-step `kbase`; the steady-state loop advances them by one k-step per step
  // (one 64-bit add per load) instead of forming base + offset each time.
  int kbase = 0;
  auto stage_slot = [&](bf16x8* stage, int n) {
    return lds_offset(stage + (n < QI ? 0 : BM * 4) + (wave * (16 * QI) + (n % QI) * 16) * 4);
  };
  // load n (0 .. 2 QI - 1) of this wavefront for k-step kt: A rows first, then B rows
  auto issue_one = [&](bf16x8* stage, int kt, int n) {
    load_to_lds_16(gp[n] + (kt - kbase) * BK, stage_slot(stage, n));
  };
  // the same for the k-step gp[n] points at, which then moves on by one
  auto issue_next = [&](bf16x8* stage, int n) {
    load_to_lds_16(gp[n], stage_slot(stage, n));
    gp[n] += BK;
  };
  auto issue = [&](bf16x8* stage, int kt) {
#pragma unroll
    for (int n = 0; n < 2 * QI; ++n) issue_one(stage, kt, n);
  };

  floatx16 acc[4][TJ];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < TJ; ++j) acc[i][j] = floatx16{};

  // Fragments of one 16-wide k-slice: 4 row tiles of A, 2 token tiles of B.
  struct Frag { bf16x8 a[4], b[TJ]; };
  auto read_frag = [&](const bf16x8* stage, int ks, Frag& f) {
    const bf16x8* As = stage;
    const bf16x8* Bs = stage + BM * 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) f.a[i] = As[swz4(wm * 128 + i * 32 + j32, ks * 2 + h)];
#pragma unroll
    for (int j = 0; j < TJ; ++j) f.b[j] = Bs[swz4(wn * (32 * TJ) + j * 32 + j32, ks * 2 + h)];
  };
  auto mfma_frag = [&](const Frag& f) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < TJ; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[i], f.b[j], acc[i][j], 0, 0, 0);
  };

  const int nk = a.d / BK;
  Frag cur, nxt;
  // One k-step.  On entry stage kt is complete and visible to everybody and `cur` holds its
  // first k-slice.  The barrier at the top publishes stage kt+1 (each wavefront first waits
  // for its own 4 loads of it; the 4 of stage kt+2 may stay in flight) and tells that everybody
  // has left stage kt-1, which is then refilled with k-step kt+3.  Because stage kt+1 is
  // already visible, its first k-slice is fetched under the last multiplies of stage kt.
  //
  // Steady-state form (kt + 3 < nk): no conditionals, so the step is one basic block, and the
  // fragment reads sit in the middle of a run of multiplies: the compiler cannot see through
  // the hand-written barrier and load statements and waits for every outstanding LDS read
  // before the first multiply that follows them, so each batch of reads is issued when the
  // previous batch has long returned and four multiplies ahead of its first use.
  auto mfma_pair = [&](const Frag& f, int i) {
#pragma unroll
    for (int j = 0; j < TJ; ++j)
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[i], f.b[j], acc[i][j], 0, 0, 0);
  };
  auto step_steady = [&](const bf16x8* st_cur, const bf16x8* st_next, bf16x8* refill) {
    __builtin_amdgcn_sched_barrier(0);  // the multiplies of the previous step stay in front of the barrier
    wait_newer<2 * QI>();
    lds_barrier();
    mfma_pair(cur, 0);
    issue_next(refill, 0);
    mfma_pair(cur, 1);
    __builtin_amdgcn_sched_barrier(0);
    read_frag(st_cur, 1, nxt);
    issue_next(refill, 1);
    __builtin_amdgcn_sched_barrier(0);
    mfma_pair(cur, 2);
    issue_next(refill, 2);
    mfma_pair(cur, 3);
    issue_next(refill, 3);
#pragma unroll
    for (int n = 4; n < 2 * QI; ++n) issue_next(refill, n);
    __builtin_amdgcn_sched_barrier(0);
    mfma_pair(nxt, 0);
    mfma_pair(nxt, 1);
    __builtin_amdgcn_sched_barrier(0);
    read_frag(st_next, 0, cur);
    __builtin_amdgcn_sched_barrier(0);
    mfma_pair(nxt, 2);
    mfma_pair(nxt, 3);
  };
  // General form for the last steps of the k loop (nothing left to refill, no next stage).
  auto step = [&](const bf16x8* st_cur, const bf16x8* st_next, bf16x8* refill, int kt) {
    if (kt + 2 < nk) wait_newer<2 * QI>();
    else wait_newer<0>();
    lds_barrier();
    read_frag(st_cur, 1, nxt);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (kt + 3 < nk && i < 2 * QI) issue_one(refill, kt + 3, i);
      mfma_pair(cur, i);
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int n = 4; n < 2 * QI; ++n)
      if (kt + 3 < nk) issue_one(refill, kt + 3, n);
    if (kt + 1 < nk) read_frag(st_next, 0, cur);
    mfma_frag(nxt);
  };

  issue(st0, 0);
  if (1 < nk) issue(st1, 1);
  if (2 < nk) issue(st2, 2);
  if (2 < nk) wait_newer<4 * QI>();
  else if (1 < nk) wait_newer<2 * QI>();
  else wait_newer<0>();
  lds_barrier();
  read_frag(st0, 0, cur);
  int kt = 0;
  if (6 < nk) {  // the steady loop refills k-step kt + 3: point the loads there
#pragma unroll
    for (int n = 0; n < 2 * QI; ++n) gp[n] += 3 * BK;
    kbase = 3;
  }
  for (; kt + 6 < nk; kt += 4) {  // all four steps refill: kt + 3 + 3 < nk
    step_steady(st0, st1, st3);
    step_steady(st1, st2, st0);
    step_steady(st2, st3, st1);
    step_steady(st3, st0, st2);
    kbase += 4;
  }
  for (; kt < nk; kt += 4) {
    step(st0, st1, st3, kt);
    if (kt + 1 < nk) step(st1, st2, st0, kt + 1);
    if (kt + 2 < nk) step(st2, st3, st1, kt + 2);
    if (kt + 3 < nk) step(st3, st0, st2, kt + 3);
  }

  // Epilogue, straight from the accumulators.  D layout of the 32x32 MFMA: lane holds
  // D[8 (r/4) + 4 h + r%4][j32], r = 0..15, so for a fixed r the 32 lanes of a half-wavefront hold
  // 32 consecutive tokens of one row: a dword store writes two full 128-byte lines, and the
  // (max, sum exp) over the wavefront's 64 tokens is a reduction over those 32 lanes (four DPP
  // steps inside rows of 16 lanes and one swap of the two rows).  No LDS, and no branch in the
  // interior tiles, so the 64 independent (row tile, r) chains interleave freely.
  constexpr float kLog2e = 1.4426950408889634f;
  const float sc = a.inv_tau;
  const int mw = m0 + wm * 128;  // first row of this wavefront
#pragma unroll
  for (int jp = 0; jp < TJ / 2; ++jp) {
    const int vbase = n0 + wn * (32 * TJ) + jp * 64;
    const int ptile = vbase / kTiledTn;
    const int v0 = vbase + j32, v1 = v0 + 32;
    float* lbase = a.logits + (size_t)(mw + 4 * h) * a.ldl + v0;
    float2* pbase = a.partials + (size_t)(mw + 4 * h) * a.nT + ptile;
    if (mw + 128 <= M && vbase + 64 <= a.V) {  // interior: wavefront-uniform
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        // phase by phase over the 16 accumulator indices, so that the 16 reduction chains are
        // independent neighbours in program order
        float mx[16], e[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int mr = i * 32 + 8 * (r >> 2) + (r & 3);
          const float l0 = acc[i][jp * 2][r] * sc, l1 = acc[i][jp * 2 + 1][r] * sc;
          acc[i][jp * 2][r] = l0;
          acc[i][jp * 2 + 1][r] = l1;
          float* dst = lbase + (size_t)mr * a.ldl;
          dst[0] = l0;
          dst[32] = l1;
          mx[r] = l0 > l1 ? l0 : l1;
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) mx[r] = max_ror<8>(mx[r]);
#pragma unroll
        for (int r = 0; r < 16; ++r) mx[r] = max_ror<4>(mx[r]);
#pragma unroll
        for (int r = 0; r < 16; ++r) mx[r] = max_ror<2>(mx[r]);
#pragma unroll
        for (int r = 0; r < 16; ++r) mx[r] = max_ror<1>(mx[r]);
#pragma unroll
        for (int r = 0; r < 16; ++r) e[r] = swap16(mx[r]);
#pragma unroll
        for (int r = 0; r < 16; ++r) mx[r] = mx[r] > e[r] ? mx[r] : e[r];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float mb = mx[r] * kLog2e;
          e[r] = __builtin_amdgcn_exp2f(fmaf(acc[i][jp * 2][r], kLog2e, -mb)) +
                 __builtin_amdgcn_exp2f(fmaf(acc[i][jp * 2 + 1][r], kLog2e, -mb));
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) e[r] += row_ror<8>(e[r]);
#pragma unroll
        for (int r = 0; r < 16; ++r) e[r] += row_ror<4>(e[r]);
#pragma unroll
        for (int r = 0; r < 16; ++r) e[r] += row_ror<2>(e[r]);
#pragma unroll
        for (int r = 0; r < 16; ++r) e[r] += row_ror<1>(e[r]);
        float t[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) t[r] = swap16(e[r]);
        // every lane of a half-wavefront holds its row's pair and writes it to the same address
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int mr = i * 32 + 8 * (r >> 2) + (r & 3);
          pbase[(size_t)mr * a.nT] = make_float2(mx[r], e[r] + t[r]);
        }
      }
    } else if (vbase < a.V) {  // edge tiles: rows past M and tokens past V are masked
      const bool ok0 = v0 < a.V, ok1 = v1 < a.V;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int mr = i * 32 + 8 * (r >> 2) + (r & 3);
          const bool row_ok = mw + 4 * h + mr < M;
          const float l0 = acc[i][jp * 2][r] * sc, l1 = acc[i][jp * 2 + 1][r] * sc;
          float* dst = lbase + (size_t)mr * a.ldl;
          if (row_ok && ok0) dst[0] = l0;
          if (row_ok && ok1) dst[32] = l1;
          float mx = row16_max(fmaxf(ok0 ? l0 : -INFINITY, ok1 ? l1 : -INFINITY));
          mx = fmaxf(mx, swap16(mx));  // finite: token vbase itself is valid
          const float mb = mx * kLog2e;
          float e = (ok0 ? exp2f(fmaf(l0, kLog2e, -mb)) : 0.f) + (ok1 ? exp2f(fmaf(l1, kLog2e, -mb)) : 0.f);
          e = row16_sum(e);
          e += swap16(e);
          if (j32 == 0 && row_ok) pbase[(size_t)mr * a.nT] = make_float2(mx, e);
        }
      }
    }
  }
}

}  // namespace

hipError_t launch_head_tiled256(const HeadArgs& a) {
  const int M = a.nrows;
  const int m_tiles = (M + BM - 1) / BM, n_tiles = (a.V + BN - 1) / BN;
  const long grid = 8L * ((n_tiles + 7) / 8) * m_tiles;
  FEF_LAUNCH_HEAD(head_tiled256_kernel<2>, dim3((unsigned)grid), dim3(512), a, a, m_tiles, n_tiles);
  return hipGetLastError();
}

}  // namespace fef
