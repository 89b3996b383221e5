// Vocabulary-head kernel for 32 < M <= 128 rows through the head, W streamed straight into
// registers.
//
// At these sizes the pass over W is the cost, and what holds the LDS-tiled kernels back is not the
// arithmetic but getting W through LDS: every direct-to-LDS load instruction costs its wavefront
// issue time, and a workgroup barrier stands between a load and its use.  The kernels for M <= 32
// show that W can go from HBM into the MFMA operand registers at 0.97 of the plain-read rate; this
// kernel keeps that for up to 128 rows by turning the product round:
//
//   a workgroup owns a contiguous run of 16-token tiles which its eight wavefronts take in turn
//   (tile j of the run goes to wavefront j % 8); a wavefront computes, for one tile at a time,
//   all M rows x 16 tokens: v_mfma_f32_16x16x32_bf16 with the W tile as the A operand (lane
//   (i, g) loads 16 bytes of token row i at k = 8 g: 64 contiguous bytes per row and instruction,
//   256 with the four loads of a macro-step) and 16-row groups of H as the B operand;
//   H is what goes through LDS (it is small, every wavefront needs all of it, and it comes from
//   L2): a ring of four stages of [16 NG rows][128 k] filled by direct-to-LDS loads three
//   macro-steps ahead, one barrier per 128 columns of k;
//   W needs no barrier and no LDS: each wavefront keeps the W slabs of three macro-steps (12 KB)
//   in flight in a register ring, across tile boundaries.
//
// No sum over wavefronts: a tile ends in its wavefront's own epilogue (16-byte non-temporal stores
// of 4 consecutive tokens per lane, running (max, sum exp) per row).  The eight tiles in work at one
// time are 128 neighbouring tokens, so their logits fill whole 512-byte pieces of every row at about
// the same moment (measured: 4 us less at M = 64 than with a contiguous run per wavefront; ordinary
// stores instead of non-temporal ones cost 16 to 24 us).  At the end the eight running (max, sum exp)
// of a row are merged through LDS into one partial per (row, workgroup), as in the kernels for
// M <= 32.
//
// All vector-memory operations of the main loop (the W loads into registers and the H loads into
// LDS) are inline assembly and share the wavefront's in-order counter; every wait is written by
// hand as "at most N younger operations outstanding".  A wait on a register load is tied to the
// registers it releases (the wait statement takes them as in/out operands), so the multiplies
// cannot move above it.  Wavefronts whose run is shorter than the workgroup's longest keep issuing
// loads (of an address that hits in cache) so that the counts hold for everybody.
//
// The compiler takes a value loaded this way to exist from the load statement on.  That is sound as
// long as it never copies such a value before the wait, i.e. as long as every multiply reads its W
// operand from the very registers a load statement wrote; the build checks the generated assembly
// for exactly this and fails otherwise.  (The kernels for M <= 32 show what happens when it does
// not hold: there, loop-carried buffers filled by assembly loads were shuffled at the loop head,
// before their wait; they use plain loads, which the compiler counts itself.)
#include <type_traits>

#include "head_common.hpp"

namespace fef {
namespace {
constexpr int kRsWaves = 8;
constexpr int kRsTurn = 4;
constexpr int kRsKm = 128;   // k columns per macro-step: four MFMA k-steps of 32

// 16 bytes per lane from gptr + OFS bytes into w; completion is waited for by hand.
template <int OFS>
__device__ inline void load_w16(bf16x8& w, const void* gptr) {
  asm volatile("global_load_dwordx4 %0, %1, off offset:%2" : "=&v"(w) : "v"(gptr), "n"(OFS) : "memory");
}
// Wait until at most N vector-memory operations younger than the wanted ones are outstanding;
// the four registers of a macro-step's slab pass through, so their users stay behind the wait.
template <int N>
__device__ inline void wait_slab(bf16x8& w) {
  asm volatile("s_waitcnt vmcnt(%1)" : "+v"(w) : "n"(N) : "memory");
}

// NG = 16-row groups of H (M <= 16 NG), even.  RW = W slabs of a wavefront's register ring, RH = H
// stages in LDS; a slab / stage is requested RW - 1 / RH - 1 macro-steps before its use.  The main loop
// takes kRsTurn macro-steps per turn: the ring sizes divide it (static ring positions) and it divides
// d / 128.  (Rings of 8 in turns of 8 were measured 3.5 % slower at M = 64 than rings of 4 in turns of
// 4, 203 to 205 us against 198; the depth of the rings made no difference.)
template <int NG, int RW, int RH>
__global__ __launch_bounds__(512) void head_rowstream_kernel(HeadArgs a, int tiles_total) {
  static_assert(NG % 2 == 0 && NG <= 8, "H stage: 4 rows per load instruction, 8 wavefronts");
  static_assert(kRsTurn % RW == 0 && kRsTurn % RH == 0, "static ring positions");
  constexpr int LW = RW - 1, LH = RH - 1;
  constexpr int ROWS = 16 * NG;
  constexpr int STAGE = ROWS * 16;           // 16-byte chunks per H stage: 256 bytes per row
  constexpr int HQ = NG / 2;                 // H load instructions per wavefront and stage
  constexpr int PER_STEP = HQ + 4;           // vector-memory operations a wavefront issues per macro-step
  __shared__ bf16x8 ringH[RH * STAGE];       // NG = 8: 32 KB per stage
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int i16 = lane & 15, g = lane >> 4;
  const int M = a.nrows;
  const int nkm = a.d / kRsKm;               // macro-steps per tile; a multiple of kRsTurn (launcher)

  // the workgroup's run of tiles; this wavefront takes tiles t_begin, t_begin + 8, ... (cnt of them)
  constexpr int ts = kRsWaves;
  const int wg_begin = (int)((long)blockIdx.x * tiles_total / gridDim.x);
  const int wg_end = (int)((long)(blockIdx.x + 1) * tiles_total / gridDim.x);
  const int t_begin = wg_begin + wave;
  const int cnt = t_begin < wg_end ? (wg_end - t_begin + ts - 1) / ts : 0;
  const int n_iter = (wg_end - wg_begin + ts - 1) / ts;  // the longest of the eight

  // H loads: instruction q of this wavefront fills rows 4 (HQ wave + q) .. + 3 of a stage; lane l
  // owns slot (row + l / 16, position l % 16) and fetches the chunk the swizzle keeps there.
  const __bf16* hp[HQ];
#pragma unroll
  for (int q = 0; q < HQ; ++q) {
    const int row = (wave * HQ + q) * 4 + (lane >> 4);
    const int c = (lane & 15) ^ (row & 15);
    hp[q] = h_row(a, min(row, M - 1)) + c * 8;  // rows past M re-read the last row; masked in the epilogue
  }
  const uint32_t slotH = lds_offset(ringH + wave * HQ * 4 * 16);
  constexpr uint32_t kStageBytes = STAGE * 16;
  // Every row of W starts at a multiple of 2 d bytes, so workgroups that walk k from 0 in step ask
  // HBM for the same low address bits at the same moment and crowd the same channels: each
  // workgroup starts its walk at another macro-step and wraps round (H and W alike).
  const int km0 = (int)((blockIdx.x * 37u) % (unsigned)nkm);
  int h_km = km0;  // macro-step (within a tile) of the next H stage to request
  // (one write of M0 for the HQ loads of a stage, with the loads told apart by their instruction offset,
  // is worth 2 to 3 % in the LDS-tiled kernels; here it measured 1 % slower and is not used)
  auto issue_h = [&](int stage) {
#pragma unroll
    for (int q = 0; q < HQ; ++q) load_to_lds_16(hp[q] + h_km * kRsKm, slotH + stage * kStageBytes + q * 1024);
    h_km = h_km + 1 == nkm ? 0 : h_km + 1;
  };

  // W loads: the prefetch position runs ahead of the multiplies over the tiles of this run; once
  // nothing is left it stays on one 256-byte piece of the first tile (loads that keep the count of
  // outstanding operations the same for every wavefront, and cost no HBM traffic).
  const __bf16* Wl = (const __bf16*)a.W + g * 8;
  auto row_base = [&](int t) { return Wl + (size_t)min(t * 16 + i16, a.V - 1) * a.d; };
  int pf_tile = 0, pf_steps = 0, pf_km = km0;  // tile of the run, steps done in it, macro-step inside the row
  int w_step = cnt > 0 ? kRsKm : 0;            // elements the position advances per macro-step
  const __bf16* wp = row_base(t_begin) + km0 * kRsKm;
  bf16x8 wbuf[RW][4];
  auto issue_w = [&](bf16x8(&slab)[4]) {
    load_w16<0>(slab[0], wp);
    load_w16<64>(slab[1], wp);
    load_w16<128>(slab[2], wp);
    load_w16<192>(slab[3], wp);
    wp += w_step;
    if (++pf_km == nkm) {  // wrap to the start of the row
      pf_km = 0;
      wp -= w_step ? a.d : 0;
    }
    if (++pf_steps == nkm) {
      pf_steps = 0;
      ++pf_tile;
      pf_km = km0;
      w_step = pf_tile < cnt ? kRsKm : 0;
      wp = row_base(pf_tile < cnt ? t_begin + pf_tile * ts : t_begin) + km0 * kRsKm;
    }
  };

  floatx4 acc[NG];
  float run_m[NG], run_s[NG];
#pragma unroll
  for (int n = 0; n < NG; ++n) {
    acc[n] = floatx4{0.f, 0.f, 0.f, 0.f};
    run_m[n] = -INFINITY;
    run_s[n] = 0.f;
  }

  // fragment of H for row group n at k-step s of a stage: row 16 n + i16, chunk 4 s + g
  auto read_h = [&](const bf16x8* stage, int s, bf16x8(&hf)[NG]) {
#pragma unroll
    for (int n = 0; n < NG; ++n) hf[n] = stage[(16 * n + i16) * 16 + ((4 * s + g) ^ i16)];
  };

  // One macro-step g with compile-time position J = g mod U.  A wavefront issues, per
  // macro-step, first the H loads of step g + LH, then the W slab of step g + LW; so when step g
  // begins, the operations younger than its H loads number 4 + (LH - 1) PER_STEP, and after this
  // step's own loads those younger than element s of its W slab number (3 - s) + LW PER_STEP.
  auto macro_step = [&](auto jc) {
    constexpr int J = decltype(jc)::value;
    const bf16x8* stage = ringH + (J % RH) * STAGE;
    bf16x8(&slab)[4] = wbuf[J % RW];
    wait_newer<4 + (LH - 1) * PER_STEP>();  // H(g) of this wavefront has landed
    lds_barrier();                          // ... and everybody's; the stage of step g - 1 has been read by all
    issue_h((J + LH) % RH);
    issue_w(wbuf[(J + LW) % RW]);
    bf16x8 hf0[NG], hf1[NG];
    read_h(stage, 0, hf0);
    wait_slab<LW * PER_STEP + 3>(slab[0]);
    read_h(stage, 1, hf1);
#pragma unroll
    for (int n = 0; n < NG; ++n) acc[n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(slab[0], hf0[n], acc[n], 0, 0, 0);
    wait_slab<LW * PER_STEP + 2>(slab[1]);
    read_h(stage, 2, hf0);
#pragma unroll
    for (int n = 0; n < NG; ++n) acc[n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(slab[1], hf1[n], acc[n], 0, 0, 0);
    wait_slab<LW * PER_STEP + 1>(slab[2]);
    read_h(stage, 3, hf1);
#pragma unroll
    for (int n = 0; n < NG; ++n) acc[n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(slab[2], hf0[n], acc[n], 0, 0, 0);
    wait_slab<LW * PER_STEP>(slab[3]);
#pragma unroll
    for (int n = 0; n < NG; ++n) acc[n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(slab[3], hf1[n], acc[n], 0, 0, 0);
  };

  // prologue, in the order of the steady state: step j issues H(j + LH) and W(j + LW)
  static_assert(LW >= LH, "the W ring is the deeper one");
#pragma unroll
  for (int j = -LW; j < 0; ++j) {
    if (j + LH >= 0) issue_h((j + LH) % RH);
    issue_w(wbuf[(j + LW) % RW]);
  }

  constexpr float kLog2e = 1.4426950408889634f;
  for (int it = 0; it < n_iter; ++it) {
    for (int km = 0; km < nkm; km += kRsTurn) {
      macro_step(std::integral_constant<int, 0>{});
      macro_step(std::integral_constant<int, 1>{});
      macro_step(std::integral_constant<int, 2>{});
      macro_step(std::integral_constant<int, 3>{});
    }
    // epilogue of tile `it` of this run: lane (i16, g) holds tokens 4 g .. 4 g + 3 of row 16 n + i16
    if (it < cnt) {
      const int v = (t_begin + it * ts) * 16 + 4 * g;
#pragma unroll
      for (int n = 0; n < NG; ++n) {
        const int row = 16 * n + i16;
        const floatx4 l = acc[n] * a.inv_tau;
        acc[n] = floatx4{0.f, 0.f, 0.f, 0.f};
        const bool row_ok = row < M;
        if (row_ok) {
          float* dst = a.logits + (size_t)row * a.ldl + v;
          if (v + 3 < a.V) {
            __builtin_nontemporal_store(l, reinterpret_cast<floatx4*>(dst));
          } else {
#pragma unroll
            for (int c = 0; c < 4; ++c)
              if (v + c < a.V) dst[c] = l[c];
          }
        }
        float mx = -INFINITY;
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if (v + c < a.V) mx = fmaxf(mx, l[c]);
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));  // finite: the tile's first token exists
        const float mb = mx * kLog2e;
        float e = 0.f;
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if (v + c < a.V) e += exp2f(fmaf(l[c], kLog2e, -mb));
        e += __shfl_xor(e, 16, 64);
        e += __shfl_xor(e, 32, 64);
        if (mx > run_m[n]) {
          run_s[n] = run_s[n] * exp2f((run_m[n] - mx) * kLog2e) + e;
          run_m[n] = mx;
        } else {
          run_s[n] += e * exp2f((mx - run_m[n]) * kLog2e);
        }
      }
    } else {
#pragma unroll
      for (int n = 0; n < NG; ++n) acc[n] = floatx4{0.f, 0.f, 0.f, 0.f};
    }
  }
  wait_newer<0>();  // the loads that ran ahead of the last tile

  // one partial per (row, workgroup): the eight running pairs of a row meet in LDS (the H ring is
  // free once every wavefront has left the main loop; a wavefront without tiles brings no mass)
  lds_barrier();
  float2* mrg = reinterpret_cast<float2*>(ringH);  // [kRsWaves][ROWS]
  if (g == 0) {
#pragma unroll
    for (int n = 0; n < NG; ++n) mrg[wave * ROWS + 16 * n + i16] = make_float2(run_m[n], run_s[n]);
  }
  lds_barrier();
  if (tid < ROWS && tid < M) {
    float2 p[kRsWaves];
    float mx = -INFINITY;
#pragma unroll
    for (int w = 0; w < kRsWaves; ++w) {
      p[w] = mrg[w * ROWS + tid];
      mx = fmaxf(mx, p[w].x);
    }
    float sum = 0.f;  // mx is finite: the workgroup has at least one tile
#pragma unroll
    for (int w = 0; w < kRsWaves; ++w) sum += p[w].y * exp2f((p[w].x - mx) * kLog2e);
    a.partials[(size_t)tid * a.nT + blockIdx.x] = make_float2(mx, sum);
  }
}

}  // namespace

bool rowstream_supports(int M, int d) { return M > 0 && M <= 128 && d % (kRsKm * kRsTurn) == 0; }

int rowstream_grid(int V) {
  const int tiles = (V + kSkinnyUnit - 1) / kSkinnyUnit;
  const int want = (tiles + kRsWaves - 1) / kRsWaves;
  return want < kSkinnyMaxGrid ? want : kSkinnyMaxGrid;
}

hipError_t launch_head_rowstream(const HeadArgs& a) {
  if (a.labels) return hipErrorInvalidValue;  // the cross-entropy epilogue is not written for this kernel
  const int tiles = (a.V + kSkinnyUnit - 1) / kSkinnyUnit;
  const int grid = rowstream_grid(a.V);
  if (a.nrows <= 64) FEF_LAUNCH_HEAD((head_rowstream_kernel<4, 4, 4>), dim3(grid), dim3(512), a, a, tiles);
  else if (a.nrows <= 96) FEF_LAUNCH_HEAD((head_rowstream_kernel<6, 4, 4>), dim3(grid), dim3(512), a, a, tiles);
  else FEF_LAUNCH_HEAD((head_rowstream_kernel<8, 4, 4>), dim3(grid), dim3(512), a, a, tiles);
  return hipGetLastError();
}

}  // namespace fef
