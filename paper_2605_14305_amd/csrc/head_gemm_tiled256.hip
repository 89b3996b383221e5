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
constexpr int kStageChunks = (BM + BN) * 4;  // 16-byte chunks per stage: A rows then B rows
constexpr int kEpiStride = 68;               // floats per staged row (64 + pad)

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
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
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
  // load n (0 .. 2 QI - 1) of this wavefront for k-step kt: A rows first, then B rows
  auto issue_one = [&](bf16x8* stage, int kt, int n) {
    const int q = n % QI;
    bf16x8* dst = stage + (n < QI ? 0 : BM * 4) + (wave * (16 * QI) + q * 16) * 4;
    load_to_lds_16(gp[n] + kt * BK, lds_offset(dst));
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
  auto step = [&](const bf16x8* st_cur, const bf16x8* st_next, bf16x8* refill, int kt) {
    if (kt + 2 < nk) wait_newer<2 * QI>();
    else wait_newer<0>();
    lds_barrier();
    read_frag(st_cur, 1, nxt);
    // The refill loads are spread between the multiplies: a wavefront issues in order, and eight
    // wavefronts pushing all their loads right after the barrier fill the address FIFO and stall
    // in front of their own MFMAs.
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (kt + 3 < nk && i < 2 * QI) issue_one(refill, kt + 3, i);
#pragma unroll
      for (int j = 0; j < TJ; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur.a[i], cur.b[j], acc[i][j], 0, 0, 0);
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
  for (int kt = 0; kt < nk; kt += 4) {
    step(st0, st1, st3, kt);
    if (kt + 1 < nk) step(st1, st2, st0, kt + 1);
    if (kt + 2 < nk) step(st2, st3, st1, kt + 2);
    if (kt + 3 < nk) step(st3, st0, st2, kt + 3);
  }
  lds_barrier();  // everybody is done with the operand stages; st0..st2 become epilogue scratch

  // Epilogue.  D layout of the 32x32 MFMA: lane holds D[8 (r/4) + 4 h + r%4][j32], r = 0..15.
  // Each wavefront stages 32 rows x 64 tokens at a time in its own scratch region.
  float* scratch = reinterpret_cast<float*>(wave < 3 ? st0 : wave < 6 ? st1 : st2) + (wave % 3) * (32 * kEpiStride);
  const int c4 = (lane & 15) * 4, rsub = lane >> 4;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
#pragma unroll
    for (int jp = 0; jp < TJ / 2; ++jp) {
      const int vbase = n0 + wn * (32 * TJ) + jp * 64;
      const int ptile = vbase / kTiledTn;
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          scratch[(8 * (r >> 2) + 4 * h + (r & 3)) * kEpiStride + j * 32 + j32] = acc[i][jp * 2 + j][r] * a.inv_tau;
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
