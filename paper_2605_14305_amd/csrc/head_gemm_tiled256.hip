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

// TJ = 32-token tiles per wavefront: 2 -> eight wavefronts of 128 x 64.  (4 -> four wavefronts of
// 128 x 128, one per SIMD, was measured slower and is not instantiated.)
template <int TJ, bool CE>
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
  if (m0 + wm * 128 >= M) {
    // None of this wavefront's 128 rows exists (the last row tile of a launch whose M is no
    // multiple of 256): it keeps its share of the loads and every barrier, in the order of the
    // steps below, and multiplies nothing.
    auto idle_step = [&](bf16x8* refill, int kt) {
      if (kt + 2 < nk) wait_newer<2 * QI>();
      else wait_newer<0>();
      lds_barrier();
      if (kt + 3 < nk) issue(refill, kt + 3);
    };
    for (int kt = 0; kt < nk; kt += 4) {
      idle_step(st3, kt);
      if (kt + 1 < nk) idle_step(st0, kt + 1);
      if (kt + 2 < nk) idle_step(st1, kt + 2);
      if (kt + 3 < nk) idle_step(st2, kt + 3);
    }
    return;
  }
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

  // Epilogue: logits and per-row (max, sum exp) partials straight from the accumulators.
  static_assert(TJ == 2, "the epilogue covers 64 tokens per wavefront");
  store_logits_and_partials<4, CE>(a, acc, m0 + wm * 128, n0 + wn * 64, M, lane);
}

}  // namespace

hipError_t launch_head_tiled256(const HeadArgs& a) {
  const int M = a.nrows;
  const int m_tiles = (M + BM - 1) / BM, n_tiles = (a.V + BN - 1) / BN;
  const long grid = 8L * ((n_tiles + 7) / 8) * m_tiles;
  if (a.labels)
    FEF_LAUNCH_HEAD((head_tiled256_kernel<2, true>), dim3((unsigned)grid), dim3(512), a, a, m_tiles, n_tiles);
  else
    FEF_LAUNCH_HEAD((head_tiled256_kernel<2, false>), dim3((unsigned)grid), dim3(512), a, a, m_tiles, n_tiles);
  return hipGetLastError();
}

}  // namespace fef
