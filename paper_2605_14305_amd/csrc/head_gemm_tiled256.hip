// Vocabulary-head kernel for large M = 2*B*K (the batched configurations).
//
// Workgroup tile 256 (rows of H) x 256 (tokens), eight wavefronts in a 2 x 4 grid, each 128 x 64 as
// 4 x 2 v_mfma_f32_32x32x16_bf16 tiles (128 accumulator registers), k-steps of 64.
//
// Operand slabs go HBM/L2 -> LDS directly (global_load_lds_dwordx4: lane l of a wavefront deposits
// its 16 bytes at LDS base + 16 l): no register staging and no ds_write in the main loop.  A row
// of a stage is 128 bytes, so one load instruction fetches eight rows of 128 contiguous bytes
// (whole L2 lines; 64-byte segments move at about 60 % of that rate out of L2), and there is one
// workgroup barrier per 64 columns of k.  The loads are inline assembly with hand-counted vmcnt
// before each barrier: with the builtin, the compiler's wait-count pass ties the fragment reads of
// one stage to the loads in flight for the others.
//
// LDS (all 160 KB of the CU): H ring of two 32 KB stages, W ring of three.  H comes from L2 / the
// Infinity Cache and is requested one k-step ahead; W comes from HBM and is requested two ahead.
// A stage is [256 rows][8 chunks of 16 B]; the LDS has 64 four-byte banks, i.e. two such rows per
// sweep, so chunk c of row r is kept at position c ^ ((r >> 1) & 7) and the 16-byte fragment
// reads of 16 consecutive rows touch every bank once.  The permutation is applied on the global
// side of the load (lane l lands at LDS base + 16 l and fetches the chunk that belongs there).
//
// One k-step is four 16-wide slices (the four H loads of a wavefront go out as one group in the
// first, the four W loads in the third).  The fragments of a slice are read, one after each multiply,
// while the multiplies of the slice before it run; the last slice of a step is multiplied after the next step's barrier,
// under the first fragment reads of the new stage, so the barrier does not idle the matrix unit
// for the latency of those reads.
//
// The epilogue works straight from the accumulator registers: for a fixed accumulator index the 32
// lanes of a half-wavefront hold 32 consecutive tokens of one row, so dword stores write whole
// 128-byte lines, and the per-row (max, sum exp) over the wavefront's 64 tokens is reduced by DPP.
//
// Tile order: workgroup ids go round-robin over the 8 XCDs; within an XCD consecutive workgroups
// take the row tiles of one token tile, so a W tile comes from HBM once and is shared through
// that XCD's L2.
#include <type_traits>

#include "head_common.hpp"

namespace fef {
namespace {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int kStage = BM * 8;   // 16-byte chunks per operand stage (BM == BN)
constexpr int kRingH = 2, kRingW = 3;

// Epilogue of a wavefront that holds a whole 128 x 128 tile (four wavefronts per workgroup), interior tiles only:
// rows mw .. mw + 127 all exist, tokens vbase .. vbase + 127 all exist.  With one wavefront per SIMD nothing else
// runs while it does, so what counts is the number of instructions, of any kind, and every wait for a result.
// Against two calls of the shared 128 x 64 epilogue: a lane holds four tokens of a row, so the first steps of a
// row's reduction are in its own registers; the reduction stops at the row of 16 lanes (the DPP steps), and each
// of the two rows of 16 that share a matrix row writes the partial of its own 64 tokens (tokens j, j + 32, j + 64,
// j + 96 of the 128, j < 16 or j >= 16: any split of the tile's tokens will do for the merge that follows), so
// nothing crosses between the rows of 16 and nothing waits for the LDS crossbar; one running pointer per row for
// the four stores; the wait states of the DPP steps paid once per eight.
// lp: this wavefront's first partial slot in LDS, [row][4 slots] of float2; the wavefront fills two slots per row.
template <bool CE>
__device__ __forceinline__ void epilogue_128x128(const HeadArgs& a, floatx16 (&acc)[2][4][2], int mw, int vbase, int lane,
                                                 float2* lp) {
  constexpr float kLog2e = 1.4426950408889634f;
  const int j32 = lane & 31, h = lane >> 5;
  const float sc = a.inv_tau;
  if constexpr (CE) {
    // A row's label token lies in one tile of one wavefront, in one lane's accumulators.  Every lane looks up the
    // labels of two of the wavefront's 128 rows; a label that falls among this tile's 128 tokens (13 % of the
    // (wavefront, tile) pairs have one at V = 126464) is then fetched in a loop over the hits with wavefront-uniform
    // indices: the 32 x 32 accumulator tile by comparison of scalars, the element inside it likewise, and the lane
    // that holds it stores it.  (Going through all of a lane's elements with a label lookup each was a chain of
    // 64 load latencies per hit: 1850 against 1700 us per call at R = 2048, and the workgroups of an XCD, which
    // share their operand tiles through its L2 while they walk in step, fell out of step: 47 % L2 hits against 77 %.)
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const int lab = a.labels[mw + q * kWave + lane];
      unsigned long long hits = __builtin_amdgcn_ballot_w64((unsigned)(lab - vbase) < 128u);
      while (hits != 0) {  // wavefront-uniform
        const int src = __builtin_ctzll(hits);
        hits &= hits - 1;
        const int rowl = q * kWave + src;                                     // row inside the wavefront's tile
        const int col = __builtin_amdgcn_readlane(lab, src) - vbase;          // token inside it
        const int ti = rowl >> 5, x = rowl & 31, th = (x >> 2) & 1, tr = ((x >> 3) << 2) | (x & 3);
        const int tc = col >> 5, tj = col & 31;
        float v = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int c = 0; c < 4; ++c)
            if (i == ti && c == tc) {  // wavefront-uniform: one of the accumulator tiles
              v = acc[c >> 1][i][c & 1][0];
#pragma unroll
              for (int r = 1; r < 16; ++r) v = r == tr ? acc[c >> 1][i][c & 1][r] : v;
            }
        if (lane == tj + 32 * th) a.label_logit[mw + rowl] = v * sc;
      }
    }
  }
  float2* pw = lp + 4 * h * 4 + ((lane >> 4) & 1);
  // Each phase runs over eight rows before the next begins (the scheduling barriers keep it so: left alone, the
  // compiler finishes one row's chain before it starts the next, every step waiting for the one before), so
  // neighbours in program order never depend on one another.
#pragma unroll
  for (int g = 0; g < 8; ++g) {
    const int i = g >> 1, r0 = (g & 1) * 8;  // 32-row tile, first accumulator index
    const int mr0 = i * 32 + 8 * (r0 >> 2);  // row of index r0 (before the 4 h of the half-wavefront)
    float l[8][4], m[8], e[8], t[8];  // t: -max log2(e)
#pragma unroll
    for (int q = 0; q < 8; ++q)
#pragma unroll
      for (int c = 0; c < 4; ++c) l[q][c] = acc[c >> 1][i][c & 1][r0 + q] * sc;
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (!CE) {
      // non-temporal, as in the shared epilogue; the pointer walks down the rows (the empty statement keeps it
      // a running pointer: one 64-bit addition per row)
      typedef __attribute__((address_space(1))) float gfloat;
      gfloat* dst = (gfloat*)(a.logits + (size_t)(mw + 4 * h + mr0) * a.ldl + vbase + j32);
      const size_t s1 = (size_t)a.ldl, s5 = 5 * (size_t)a.ldl;
#pragma unroll
      for (int q = 0; q < 8; ++q) {
#pragma unroll
        for (int c = 0; c < 4; ++c) __builtin_nontemporal_store(l[q][c], dst + 32 * c);
        if (q < 7) {
          dst += q == 3 ? s5 : s1;
          asm("" : "+v"(dst));
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) m[q] = vmax3(l[q][0], l[q][1], vmax(l[q][2], l[q][3]));
    __builtin_amdgcn_sched_barrier(0);
    max_ror_x8<8>(m);
    max_ror_x8<4>(m);
    max_ror_x8<2>(m);
    max_ror_x8<1>(m);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < 8; ++q) t[q] = m[q] * -kLog2e;
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
#pragma unroll
      for (int q = 0; q < 8; ++q) l[q][c] = fmaf(l[q][c], kLog2e, t[q]);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int q = 0; q < 8; ++q) l[q][c] = __builtin_amdgcn_exp2f(l[q][c]);
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) e[q] = (l[q][0] + l[q][1]) + (l[q][2] + l[q][3]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < 8; ++q) e[q] += row_ror<8>(e[q]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < 8; ++q) e[q] += row_ror<4>(e[q]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < 8; ++q) e[q] += row_ror<2>(e[q]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < 8; ++q) e[q] += row_ror<1>(e[q]);
    __builtin_amdgcn_sched_barrier(0);
    // every lane of a row of 16 holds the pair of its 64 tokens and writes it to the same address
#pragma unroll
    for (int q = 0; q < 8; ++q) pw[(mr0 + 8 * (q >> 2) + (q & 3)) * 4] = make_float2(m[q], e[q]);
    __builtin_amdgcn_sched_barrier(0);
  }
}

template <bool CE>
__global__ __launch_bounds__(512) void head_tiled256_kernel(HeadArgs a, int m_tiles, int n_tiles) {
  __shared__ bf16x8 ringH[kRingH * kStage];  // 64 KB
  __shared__ bf16x8 ringW[kRingW * kStage];  // 96 KB
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 2, wn = wave & 3;
  const int j32 = lane & 31, h = lane >> 5;
  const int M = a.nrows;

  const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
  const int nt = xcd + 8 * (seq / m_tiles), mt = seq % m_tiles;
  if (nt >= n_tiles) return;
  const int m0 = mt * BM, n0 = nt * BN;
  const int nk = a.d / BK;
  // Every row of W starts at a multiple of 2 d bytes, so workgroups that walk k from 0 in step ask HBM for the
  // same low address bits at the same moment: each token tile starts its walk at another k-step and wraps
  // (M = 256: head 277 -> 263 us, step 326 -> 321.5 us; with several row tiles per token tile, which share H
  // in time through L2, the same change measured +2 % at M = 2048 and is not used there).
  const int k0 = (int)((unsigned)(nt * 37) % (unsigned)nk);
  int h_left = nk - k0, w_left = nk - k0;  // steps until the walk is back at k = 0

  // Direct-to-LDS loads: wavefront w fills rows [32 w, 32 w + 32) of an H stage and of a W stage,
  // 8 rows per instruction; lane l owns LDS slot (row 8 q + l / 8, position l % 8).
  const __bf16* gh[4];
  const __bf16* gw[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int rl = wave * 32 + q * 8 + (lane >> 3);
    const int c = (lane & 7) ^ ((rl >> 1) & 7);
    const int r = min(m0 + rl, M - 1);      // rows past M / V re-read the last row; masked in the epilogue
    const int v = min(n0 + rl, a.V - 1);
    gh[q] = h_row(a, r) + c * 8 + k0 * BK;
    gw[q] = (const __bf16*)a.W + (size_t)v * a.d + c * 8 + k0 * BK;
    gh[q] -= q * 512;  // 1024 bytes per position in the group of four: the instruction offset puts them back
    gw[q] -= q * 512;
  }
  // Four loads behind one write of M0 (the instruction offset moves the LDS address and the memory
  // address alike): every write of M0 in front of a direct-to-LDS load holds the wavefront for some
  // tens of cycles; 2 writes per k-step instead of 8 are worth 2.7 % at M = 256.
  auto issue4 = [&](const __bf16* (&g)[4], uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %4\n\ts_nop 0\n\t"
                 "global_load_lds_dwordx4 %0, off\n\tglobal_load_lds_dwordx4 %1, off offset:1024\n\t"
                 "global_load_lds_dwordx4 %2, off offset:2048\n\tglobal_load_lds_dwordx4 %3, off offset:3072"
                 :: "v"(g[0]), "v"(g[1]), "v"(g[2]), "v"(g[3]), "s"(lds_base) : "memory");
#pragma unroll
    for (int q = 0; q < 4; ++q) g[q] += BK;
  };
  const uint32_t slotH = lds_offset(ringH + wave * 32 * 8), slotW = lds_offset(ringW + wave * 32 * 8);
  constexpr uint32_t kStageBytes = kStage * 16;
  // loads of this wavefront for the k-step the pointers stand at, which then move on by one step
  // single loads (prologue, wavefronts without rows)
  auto issue_h = [&](int stage, int q) {
    load_to_lds_16(gh[q] + q * 512, slotH + stage * kStageBytes + q * 1024);
    gh[q] += BK;
  };
  auto issue_w = [&](int stage, int q) {
    load_to_lds_16(gw[q] + q * 512, slotW + stage * kStageBytes + q * 1024);
    gw[q] += BK;
  };

  auto wrap_h = [&]() {  // after the H loads of a step
    if (--h_left == 0)
#pragma unroll
      for (int q = 0; q < 4; ++q) gh[q] -= a.d;
  };
  auto wrap_w = [&]() {
    if (--w_left == 0)
#pragma unroll
      for (int q = 0; q < 4; ++q) gw[q] -= a.d;
  };

  floatx16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = floatx16{};

  struct Frag { bf16x8 a[4], b[2]; };
  auto mfma_rows = [&](const Frag& f, int i0, int i1) {
#pragma unroll
    for (int i = i0; i < i1; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[i], f.b[j], acc[i][j], 0, 0, 0);
  };

  const bool idle = m0 + wm * 128 >= M;  // none of this wavefront's rows exists: loads and barriers only

  // prologue: H(0), W(0), W(1)
#pragma unroll
  for (int q = 0; q < 4; ++q) issue_h(0, q);
  wrap_h();
#pragma unroll
  for (int q = 0; q < 4; ++q) issue_w(0, q);
  wrap_w();
  if (1 < nk) {
#pragma unroll
    for (int q = 0; q < 4; ++q) issue_w(1, q);
    wrap_w();
  }

  Frag cur, nxt;
#pragma unroll
  for (int i = 0; i < 4; ++i) cur.a[i] = bf16x8{};
#pragma unroll
  for (int j = 0; j < 2; ++j) cur.b[j] = bf16x8{};  // "last slice of step -1": multiplies by zero

  // One k-step.  On entry `cur` holds the last slice of the step before.  Outstanding loads of
  // this wavefront, oldest first: H(kt) [4], W(kt+1) [4]; the barrier needs H(kt) (W(kt) is older).
  // FULL: kt + 2 < nk, every refill exists and the step is one basic block.
  auto step = [&](int kt, int sh, int sw, auto full) {
    constexpr bool FULL = decltype(full)::value;
    const bf16x8* Hs = ringH + sh * kStage;
    const bf16x8* Ws = ringW + sw * kStage;
    const int sh1 = sh ^ 1, sw2 = sw == 0 ? 2 : sw - 1;  // stages of H(kt+1) and W(kt+2)
    __builtin_amdgcn_sched_barrier(0);
    if (FULL || kt + 1 < nk) wait_newer<4>();
    else wait_newer<0>();
    lds_barrier();
    if (idle) {
      if (FULL || kt + 1 < nk) {
#pragma unroll
        for (int q = 0; q < 4; ++q) issue_h(sh1, q);
        wrap_h();
      }
      if (FULL || kt + 2 < nk) {
#pragma unroll
        for (int q = 0; q < 4; ++q) issue_w(sw2, q);
        wrap_w();
      }
      return;
    }
    // Reads dealt out one after each multiply, in the order the next slice wants them, and the group of four
    // loads after the seventh multiply of its slice: 2 to 3 % on the whole step at M = 256 against reading a
    // slice's six fragments in one run (the second wavefront of the SIMD fills such gaps only in part).
    auto read_one = [&](int ks, Frag& f, int n) {  // a0, b0, b1, a1, a2, a3
      if (n == 0) f.a[0] = Hs[swz(wm * 128 + j32, ks * 2 + h)];
      else if (n <= 2) f.b[n - 1] = Ws[swz(wn * 64 + (n - 1) * 32 + j32, ks * 2 + h)];
      else f.a[n - 2] = Hs[swz(wm * 128 + (n - 2) * 32 + j32, ks * 2 + h)];
    };
    auto slice = [&](int ks, Frag& rd, const Frag& mm, int loads) {
#pragma unroll
      for (int n = 0; n < 8; ++n) {
        const int i = n >> 1, j = n & 1;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(mm.a[i], mm.b[j], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (n < 6) {
          read_one(ks, rd, n);
          __builtin_amdgcn_sched_barrier(0);
        }
        if (n == 6) {
          if (loads == 1 && (FULL || kt + 1 < nk)) {
            issue4(gh, slotH + sh1 * kStageBytes);
            wrap_h();
          }
          if (loads == 2 && (FULL || kt + 2 < nk)) {
            issue4(gw, slotW + sw2 * kStageBytes);
            wrap_w();
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    };
    slice(0, nxt, cur, 1);
    slice(1, cur, nxt, 0);
    slice(2, nxt, cur, 2);
    slice(3, cur, nxt, 0);
  };

  int kt = 0, sw = 0;
  for (; kt + 3 < nk; kt += 2) {  // two full steps: kt + 1 + 2 < nk
    step(kt, 0, sw, std::true_type{});
    sw = sw == 2 ? 0 : sw + 1;
    step(kt + 1, 1, sw, std::true_type{});
    sw = sw == 2 ? 0 : sw + 1;
  }
  for (; kt < nk; ++kt) {
    step(kt, kt & 1, sw, std::false_type{});
    sw = sw == 2 ? 0 : sw + 1;
  }
  if (!idle) mfma_rows(cur, 0, 4);  // last slice of the last step

  lds_barrier();  // nobody reads the rings any more: the H ring takes the partials
  float2* lp = reinterpret_cast<float2*>(ringH);
  if (!idle) store_logits_and_partials<4, CE>(a, acc, m0 + wm * 128, n0 + wn * 64, M, lane, lp, wm * 128, wn);
  lds_barrier();
  merge_tile_partials(a, lp, BM, m0, nt, M, tid);
}


// ---------------------------------------------------------------------------------------------
// The same tile with FOUR wavefronts in a 2 x 2 grid, each 128 x 128 as 4 x 4 MFMA tiles (256
// accumulator registers; one wavefront per SIMD has 512 registers to itself), for M > 256.
//
// Why: with eight wavefronts of 128 x 64, a 16-wide slice of k costs every wavefront 4 + 2 fragment
// reads of 1 KB for 8 multiplies, 48 KB per CU and slice, which together with the 16 KB the loads
// deposit per slice is all the LDS can move (128 bytes per clock) in the 512 clocks the multiplies
// of a slice take: the matrix units cannot be busier than the LDS lets them.  A 128 x 128
// wavefront reads 4 + 4 fragments for 16 multiplies: 32 KB per CU and slice, three quarters of
// the LDS rate.  (At M = 256 the kernel is short of memory parallelism rather than of LDS rate and
// the eight wavefronts do better.)
//
// Loads: wavefront w fills rows [64 w, 64 w + 64) of an H stage and of a W stage (8 + 8
// instructions per k-step, four per slice).
//
// One workgroup per tile, as above.  A persistent form (one workgroup per CU walking the tiles
// b, b + G, ... and asking for the first stages of its next tile before the epilogue of the current
// one) was measured 2.5 % slower at M = 512 to 2048: the hardware's dispatch of one workgroup per
// tile balances the CUs better than a fixed share of 15 or 16 tiles each.
// ---------------------------------------------------------------------------------------------
template <bool CE>
__global__ __launch_bounds__(256) void head_tiled256w4_kernel(HeadArgs a, int m_tiles, int n_tiles) {
  __shared__ bf16x8 ringH[kRingH * kStage];  // 64 KB
  __shared__ bf16x8 ringW[kRingW * kStage];  // 96 KB
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int j32 = lane & 31, h = lane >> 5;
  const int M = a.nrows;
  const int nk = a.d / BK;

  const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
  const int nt = xcd + 8 * (seq / m_tiles), mt = seq % m_tiles;
  if (nt >= n_tiles) return;
  const int m0 = mt * BM, n0 = nt * BN;

  const __bf16* gh[8];
  const __bf16* gw[8];
  const uint32_t slotH = lds_offset(ringH + wave * 64 * 8), slotW = lds_offset(ringW + wave * 64 * 8);
  constexpr uint32_t kStageBytes = kStage * 16;
  // The pointer moves on right behind its load (the empty statement pins the addition there): left to
  // itself the compiler gathers the sixteen 64-bit additions of a step in front of the barrier, a run
  // during which the matrix unit has nothing to do.
  auto issue_h = [&](int stage, int q) {
    load_to_lds_16(gh[q], slotH + stage * kStageBytes + q * 1024);
    gh[q] += BK;
    asm volatile("" : "+v"(gh[q]));
  };
  auto issue_w = [&](int stage, int q) {
    load_to_lds_16(gw[q], slotW + stage * kStageBytes + q * 1024);
    gw[q] += BK;
    asm volatile("" : "+v"(gw[q]));
  };
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    const int rl = wave * 64 + q * 8 + (lane >> 3);
    const int c = (lane & 7) ^ ((rl >> 1) & 7);
    const int r = min(m0 + rl, M - 1);      // rows past M / V re-read the last row; masked in the epilogue
    const int v = min(n0 + rl, a.V - 1);
    gh[q] = h_row(a, r) + c * 8;
    gw[q] = (const __bf16*)a.W + (size_t)v * a.d + c * 8;
  }
  // prologue: H(0), W(0), W(1)
#pragma unroll
  for (int q = 0; q < 8; ++q) issue_h(0, q);
#pragma unroll
  for (int q = 0; q < 8; ++q) issue_w(0, q);
  if (1 < nk) {
#pragma unroll
    for (int q = 0; q < 8; ++q) issue_w(1, q);
  }

  floatx16 acc[2][4][2];  // [64-token half][32-row tile][32-token tile]
  struct Frag { bf16x8 a[4], b[4]; };
  // fragment n of slice ks in the order the next slice's multiplies want them: a0, b0, b1, b2, b3, a1, a2, a3
  auto read_one = [&](const bf16x8* Hs, const bf16x8* Ws, int ks, Frag& f, int n) {
    if (n == 0) f.a[0] = Hs[swz(wm * 128 + j32, ks * 2 + h)];
    else if (n <= 4) f.b[n - 1] = Ws[swz(wn * 128 + (n - 1) * 32 + j32, ks * 2 + h)];
    else f.a[n - 4] = Hs[swz(wm * 128 + (n - 4) * 32 + j32, ks * 2 + h)];
  };
  auto mfma_row = [&](const Frag& f, int i) {
#pragma unroll
    for (int j = 0; j < 4; ++j)
      acc[j >> 1][i][j & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[i], f.b[j], acc[j >> 1][i][j & 1], 0, 0, 0);
  };

  // none of this wavefront's rows exists: loads and barriers only (wavefront-uniform, and said so)
  const bool idle = __builtin_amdgcn_readfirstlane((int)(m0 + wm * 128 >= M)) != 0;
#pragma unroll
  for (int c = 0; c < 2; ++c)
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) acc[c][i][j] = floatx16{};
  Frag cur, nxt;
#pragma unroll
  for (int i = 0; i < 4; ++i) cur.a[i] = cur.b[i] = bf16x8{};  // "last slice of step -1": multiplies by zero

  // One k-step; outstanding loads of this wavefront on entry, oldest first: H(kt) [8], W(kt+1) [8].
  auto step = [&](int kt, int sh, int sw, auto full, auto idle_tag) __attribute__((always_inline)) {
    constexpr bool FULL = decltype(full)::value;
    constexpr bool IDLE = decltype(idle_tag)::value;
    const bf16x8* Hs = ringH + sh * kStage;
    const bf16x8* Ws = ringW + sw * kStage;
    const int sh1 = sh ^ 1, sw2 = sw == 0 ? 2 : sw - 1;
    const bool more_h = FULL || kt + 1 < nk, more_w = FULL || kt + 2 < nk;
    __builtin_amdgcn_sched_barrier(0);
    if (more_h) wait_newer<8>();
    else wait_newer<0>();
    lds_barrier();
    if constexpr (IDLE) {
      if (more_h)
#pragma unroll
        for (int q = 0; q < 8; ++q) issue_h(sh1, q);
      if (more_w)
#pragma unroll
        for (int q = 0; q < 8; ++q) issue_w(sw2, q);
      return;
    }
    // Slice s of this step is read while slice s - 1 (s = 0: the last slice of the step before) is
    // multiplied.  With one wavefront per SIMD the matrix unit has nothing to run while this wavefront
    // issues anything else, and it holds only one multiply beyond the one in work: a run of eight
    // fragment reads or four loads between two multiplies leaves it idle for the length of the run
    // (in a loop of multiplies, reads, loads and barriers only: 1837 TFLOP/s with the reads and loads
    // of a slice in runs, 2270 with one read after every second multiply and one load after the first
    // multiply of each row; multiplies alone 2460).  So everything is dealt out singly.
    auto phase = [&](int ks, Frag& rd, const Frag& mm, bool h_loads, int q0) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          acc[j >> 1][i][j & 1] =
              __builtin_amdgcn_mfma_f32_32x32x16_bf16(mm.a[i], mm.b[j], acc[j >> 1][i][j & 1], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
          if (j & 1) {
            read_one(Hs, Ws, ks, rd, i * 2 + (j >> 1));
            __builtin_amdgcn_sched_barrier(0);
          } else if (j == 0) {
            if (h_loads) {
              if (more_h) issue_h(sh1, q0 + i);
            } else {
              if (more_w) issue_w(sw2, q0 + i);
            }
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      }
    };
    phase(0, nxt, cur, true, 0);
    phase(1, cur, nxt, true, 4);
    phase(2, nxt, cur, false, 0);
    phase(3, cur, nxt, false, 4);
  };

  // Two copies of the loop, chosen once: a wavefront without rows only loads and meets the barriers.  (With
  // the choice inside the step the two paths meet again in every step, and the compiler reconciles their
  // registers there with sixteen moves in front of the barrier.)
  auto walk = [&](auto idle_tag) __attribute__((always_inline)) {
    int kt = 0, sw = 0;
    for (; kt + 3 < nk; kt += 2) {  // two full steps: kt + 1 + 2 < nk
      step(kt, 0, sw, std::true_type{}, idle_tag);
      sw = sw == 2 ? 0 : sw + 1;
      step(kt + 1, 1, sw, std::true_type{}, idle_tag);
      sw = sw == 2 ? 0 : sw + 1;
    }
    for (; kt < nk; ++kt) {
      step(kt, kt & 1, sw, std::false_type{}, idle_tag);
      sw = sw == 2 ? 0 : sw + 1;
    }
  };
  float2* lp = reinterpret_cast<float2*>(ringH);
  if (idle) {
    walk(std::true_type{});
    lds_barrier();
  } else {
    walk(std::false_type{});
#pragma unroll
    for (int i = 0; i < 4; ++i) mfma_row(cur, i);  // last slice of the last step
    lds_barrier();  // nobody reads the rings any more: the H ring takes the partials
    const int mw = m0 + wm * 128, vb = n0 + wn * 128;
    if (mw + 128 <= M && vb + 128 <= a.V) {  // wavefront-uniform
      epilogue_128x128<CE>(a, acc, mw, vb, lane, lp + wm * 128 * 4 + 2 * wn);
    } else {
      store_logits_and_partials<4, CE>(a, acc[0], mw, vb, M, lane, lp, wm * 128, 2 * wn);
      store_logits_and_partials<4, CE>(a, acc[1], mw, vb + 64, M, lane, lp, wm * 128, 2 * wn + 1);
    }
  }
  lds_barrier();
  merge_tile_partials(a, lp, BM, m0, nt, M, tid);
}

}  // namespace

hipError_t launch_head_tiled256(const HeadArgs& a) {
  const int M = a.nrows;
  const int m_tiles = (M + BM - 1) / BM, n_tiles = (a.V + BN - 1) / BN;
  const long grid = 8L * ((n_tiles + 7) / 8) * m_tiles;
  if (m_tiles == 1) {  // M <= 256: eight wavefronts of 128 x 64, one workgroup per tile
    if (a.labels)
      FEF_LAUNCH_HEAD((head_tiled256_kernel<true>), dim3((unsigned)grid), dim3(512), a, a, m_tiles, n_tiles);
    else
      FEF_LAUNCH_HEAD((head_tiled256_kernel<false>), dim3((unsigned)grid), dim3(512), a, a, m_tiles, n_tiles);
    return hipGetLastError();
  }
  // M > 256: four wavefronts of 128 x 128
  if (a.labels)
    FEF_LAUNCH_HEAD((head_tiled256w4_kernel<true>), dim3((unsigned)grid), dim3(256), a, a, m_tiles, n_tiles);
  else
    FEF_LAUNCH_HEAD((head_tiled256w4_kernel<false>), dim3((unsigned)grid), dim3(256), a, a, m_tiles, n_tiles);
  return hipGetLastError();
}

}  // namespace fef
