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
// The epilogue stages each 32 x 64 block of logits through LDS so that rows leave as 256-byte
// coalesced stores and the per-row (max, sum exp) over the wavefront's 64 tokens is reduced
// inside DPP rows of 16 lanes.
//
// Tile order: workgroup ids go round-robin over the 8 XCDs; within an XCD consecutive
// workgroups take the row tiles of one token tile, so a W tile comes from HBM once and is
// shared through that XCD's L2.
#include "head_common.hpp"

namespace fef {
namespace {

constexpr int BM = 256, BN = 256, BK = 32;
constexpr int kThreads = 512;
constexpr int kStageChunks = (BM + BN) * 4;  // 16-byte chunks per stage: A rows then B rows
constexpr int kEpiStride = 68;               // floats per staged row (64 + pad)

__device__ inline int swz4(int row, int chunk) { return row * 4 + (chunk ^ ((row >> 2) & 3)); }

__global__ __launch_bounds__(kThreads) void head_tiled256_kernel(HeadArgs a, int m_tiles, int n_tiles) {
  // one array per stage, so the compiler can tell the in-flight LDS writes of the other stages
  // from the fragment reads of the current one
  __shared__ bf16x8 st0[kStageChunks], st1[kStageChunks], st2[kStageChunks], st3[kStageChunks];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 2, wn = wave & 3;
  const int j32 = lane & 31, h = lane >> 5;
  const int M = 2 * a.BK;

  const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
  const int nt = xcd + 8 * (seq / m_tiles), mt = seq % m_tiles;
  if (nt >= n_tiles) return;
  const int m0 = mt * BM, n0 = nt * BN;

  // Direct-to-LDS loads: wavefront w fills rows [32 w, 32 w + 32) of A and of B, 16 rows per
  // instruction; lane l owns LDS slot (row 16 q + l/4, position l%4) and fetches the chunk that
  // the swizzle assigns to that slot.
  const __bf16* gp[4];
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const int rl = wave * 32 + q * 16 + (lane >> 2);       // row inside the tile
    const int c = (lane & 3) ^ ((rl >> 2) & 3);            // logical 16-byte chunk of that row
    const int r = min(m0 + rl, M - 1);                     // rows past M / V re-read the last
    const int v = min(n0 + rl, a.V - 1);                   // row; masked in the epilogue
    gp[q] = h_row(a, r) + c * 8;
    gp[2 + q] = (const __bf16*)a.W + (size_t)v * a.d + c * 8;
  }
  auto issue = [&](bf16x8* stage, int kt) {
    const int k0 = kt * BK;
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      __builtin_amdgcn_global_load_lds(gp[q] + k0, stage + (wave * 32 + q * 16) * 4, 16, 0, 0);
      __builtin_amdgcn_global_load_lds(gp[2 + q] + k0, stage + BM * 4 + (wave * 32 + q * 16) * 4, 16, 0, 0);
    }
  };

  floatx16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = floatx16{};

  auto compute = [&](const bf16x8* stage) {
    const bf16x8* As = stage;
    const bf16x8* Bs = stage + BM * 4;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 af[4], bf[2];
#pragma unroll
      for (int i = 0; i < 4; ++i) af[i] = As[swz4(wm * 128 + i * 32 + j32, ks * 2 + h)];
#pragma unroll
      for (int j = 0; j < 2; ++j) bf[j] = Bs[swz4(wn * 64 + j * 32 + j32, ks * 2 + h)];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
    }
  };

  const int nk = a.d / BK;
  // One k-step: wait for this wavefront's share of the stage (4 loads per stage; newer stages
  // may stay in flight), barrier so that everybody's share is visible and everybody has left
  // the stage that is refilled next, refill, multiply.
  auto step = [&](bf16x8* cur, bf16x8* refill, int kt) {
    if (kt + 2 < nk) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    else if (kt + 1 < nk) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    lds_barrier();
    if (kt + 3 < nk) issue(refill, kt + 3);
    compute(cur);
  };

  issue(st0, 0);
  if (1 < nk) issue(st1, 1);
  if (2 < nk) issue(st2, 2);
  for (int kt = 0; kt < nk; kt += 4) {
    step(st0, st3, kt);
    if (kt + 1 < nk) step(st1, st0, kt + 1);
    if (kt + 2 < nk) step(st2, st1, kt + 2);
    if (kt + 3 < nk) step(st3, st2, kt + 3);
  }
  lds_barrier();  // everybody is done with the operand stages; st0..st2 become epilogue scratch

  // Epilogue.  D layout of the 32x32 MFMA: lane holds D[8 (r/4) + 4 h + r%4][j32], r = 0..15.
  float* scratch = reinterpret_cast<float*>(wave < 3 ? st0 : wave < 6 ? st1 : st2) + (wave % 3) * (32 * kEpiStride);
  const int vbase = n0 + wn * 64;
  const int ptile = vbase / kTiledTn;
  const int c4 = (lane & 15) * 4, rsub = lane >> 4;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        scratch[(8 * (r >> 2) + 4 * h + (r & 3)) * kEpiStride + j * 32 + j32] = acc[i][j][r] * a.inv_tau;
    // the wavefront re-reads only its own region; LDS operations of one wavefront stay in order
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int rl = it * 4 + rsub;
      const floatx4 v4 = *reinterpret_cast<const floatx4*>(scratch + rl * kEpiStride + c4);
      const int m = m0 + wm * 128 + i * 32 + rl;
      const int v = vbase + c4;
      const bool row_ok = m < M;
      float* dst = a.logits + (size_t)m * a.ldl + v;
      float mx = -INFINITY;
      if (row_ok && v + 3 < a.V) {
        *reinterpret_cast<floatx4*>(dst) = v4;
        mx = fmaxf(fmaxf(v4[0], v4[1]), fmaxf(v4[2], v4[3]));
      } else if (row_ok) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if (v + q < a.V) { dst[q] = v4[q]; mx = fmaxf(mx, v4[q]); }
      }
      mx = row16_max(mx);
      float e = 0.f;
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (row_ok && v + q < a.V) e += __expf(v4[q] - mx);
      e = row16_sum(e);
      if ((lane & 15) == 0 && row_ok && vbase < a.V)
        a.partials[(size_t)m * a.nT + ptile] = make_float2(mx, e);
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  }
}

}  // namespace

hipError_t launch_head_tiled256(const HeadArgs& a) {
  const int M = 2 * a.BK;
  const int m_tiles = (M + BM - 1) / BM, n_tiles = (a.V + BN - 1) / BN;
  const long grid = 8L * ((n_tiles + 7) / 8) * m_tiles;
  hipExtLaunchKernelGGL(head_tiled256_kernel, dim3((unsigned)grid), dim3(kThreads), 0, a.stream,
                        a.ev_begin, a.ev_end, 0, a, m_tiles, n_tiles);
  return hipGetLastError();
}

}  // namespace fef
