// Vocabulary-head kernel for 32 < M <= 128 rows through the head (a few sequences per call, or a
// DRAFT / TARGET call of up to 16 eight-token windows).  At these sizes the pass over W is still
// the cost (2 M V d flops need well under the time 1 GB of W takes from HBM), so the kernel is
// built around streaming W without a pause.
//
// One persistent workgroup per CU takes the 256-token tiles b, b + G, ... and walks k in steps of
// 32 over all of them as ONE sequence of steps: W goes through a ring of eight 16 KB LDS stages
// filled by direct-to-LDS loads seven steps ahead (112 KB of W in flight per CU; with 64 bytes per
// row per step HBM latency under load is several microseconds), H, which every workgroup re-reads
// and which therefore sits in L2, through a ring of four 8 KB stages three steps ahead.  Together
// they use the whole 160 KB of LDS.  The loads run on across tile boundaries, so only the first
// tile of a workgroup pays the cold start, and the epilogue of a tile (registers only, no LDS)
// runs while the first stages of the next tile arrive.  The vector-memory counter of a wavefront
// completes in order, so two different leads cannot share a wavefront: wavefronts 0..3 load W
// (four 1 KB loads per step each), wavefronts 4..7 load H (two per step each).  The stores of an
// epilogue enter the same counter behind the loads in flight; the waits that follow are by count
// of the youngest operations, so they can only wait for more than they need, never for less.
//
// Eight wavefronts as 2 (64-row halves) x 4 (64-token columns), each 2 x 2
// v_mfma_f32_32x32x16_bf16 tiles over the full k: eight 16-byte fragment reads for eight
// multiplies per step, and a tile ends in the shared epilogue with no exchange between wavefronts.
//
// LDS stages are [rows][4 chunks of 16 B], chunks swizzled as in the 256 x 256 kernel.
#include <type_traits>

#include "head_common.hpp"

namespace fef {
namespace {

constexpr int SM = 128, SN = 256, SK = 32;
constexpr int kRingW = 8, kRingH = 4;          // stages; loads run kRing - 1 k-steps ahead
constexpr int kStageW = SN * 4, kStageH = SM * 4;  // 16-byte chunks per stage
constexpr int kLoadsW = 4, kLoadsH = 2;        // load instructions per loading wavefront per stage

struct Frag {
  bf16x8 a[2][2], b[2][2];  // [16-wide k-slice][32-row / 32-token tile]
};

template <bool CE>
__global__ __launch_bounds__(512) void head_stream_kernel(HeadArgs a, int n_tiles) {
  __shared__ bf16x8 ringW[kRingW * kStageW];  // 128 KB
  __shared__ bf16x8 ringH[kRingH * kStageH];  // 32 KB: one workgroup per CU
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 2, wn = wave & 3;  // row half, token column
  const int j32 = lane & 31, h = lane >> 5;
  const int M = a.nrows;
  const int G = gridDim.x;
  const int nk = a.d / SK;
  const int my_tiles = (n_tiles - (int)blockIdx.x + G - 1) / G;
  const int T = my_tiles * nk;  // steps of this workgroup; even, because nk is

  floatx16 acc[2][2];
  auto clear_acc = [&]() {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) acc[i][j] = floatx16{};
  };
  clear_acc();

  // fragment read addresses inside a stage (chunks); the stage offset is added per step
  int fa[2][2], fb[2][2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks)
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      fa[ks][i] = swz4(wm * 64 + i * 32 + j32, ks * 2 + h);
      fb[ks][i] = swz4(wn * 64 + i * 32 + j32, ks * 2 + h);
    }
  auto read_frag = [&](int sw, int sh, Frag& f) {
    const bf16x8* As = ringH + sh * kStageH;
    const bf16x8* Bs = ringW + sw * kStageW;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        f.a[ks][i] = As[fa[ks][i]];
        f.b[ks][i] = Bs[fb[ks][i]];
      }
  };
  auto mfma_row = [&](const Frag& f, int ks, int i) {
#pragma unroll
    for (int j = 0; j < 2; ++j)
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[ks][i], f.b[ks][j], acc[i][j], 0, 0, 0);
  };

  // The whole sequence of steps for one loading role.  ROLE 0: this wavefront loads W rows
  // [64 w, 64 w + 64) of every stage (lead kRingW - 1); ROLE 1: H rows [32 (w - 4), +32) (lead
  // kRingH - 1).  Lane l of a load owns LDS slot (row + l/4, position l%4) and fetches the chunk
  // the swizzle assigns to that slot.  Rows past M / V re-read the last row; they are masked in
  // the epilogue.
  auto run = [&](auto role) {
    constexpr bool W_ROLE = decltype(role)::value == 0;
    constexpr int NL = W_ROLE ? kLoadsW : kLoadsH;     // loads per stage
    constexpr int LEAD = (W_ROLE ? kRingW : kRingH) - 1;
    constexpr int RING = LEAD + 1;
    constexpr uint32_t kStageBytes = (W_ROLE ? kStageW : kStageH) * 16;
    const __bf16* gp[NL];
    uint32_t slot0[NL];  // LDS byte offset of load n in stage 0
    int lrow[NL], lchunk[NL];
#pragma unroll
    for (int n = 0; n < NL; ++n) {
      lrow[n] = (W_ROLE ? wave * 64 : (wave - 4) * 32) + n * 16 + (lane >> 2);
      lchunk[n] = ((lane & 3) ^ ((lrow[n] >> 2) & 3)) * 8;
      const bf16x8* base = W_ROLE ? ringW : ringH;
      slot0[n] = lds_offset(base + ((W_ROLE ? wave * 64 : (wave - 4) * 32) + n * 16) * 4);
    }
    // loader cursor: the next step to load is k-step kl of tile tile_l and goes to stage s_load
    int tile_l = blockIdx.x, kl = 0, s_load = 0, t_load = 0;
    auto retarget = [&]() {  // gp[] at k = 0 of tile tile_l
#pragma unroll
      for (int n = 0; n < NL; ++n)
        gp[n] = W_ROLE ? (const __bf16*)a.W + (size_t)min(tile_l * SN + lrow[n], a.V - 1) * a.d + lchunk[n]
                       : h_row(a, min(lrow[n], M - 1)) + lchunk[n];
    };
    retarget();
    auto issue_one = [&](int n) {
      load_to_lds_16(gp[n], __builtin_amdgcn_readfirstlane(slot0[n] + s_load * kStageBytes));
      gp[n] += SK;
    };
    auto loaded_step = [&]() {  // bookkeeping after the NL loads of one step
      s_load = s_load + 1 == RING ? 0 : s_load + 1;
      ++t_load;
      if (++kl == nk) {
        kl = 0;
        tile_l += G;
        if (t_load < T) retarget();
      }
    };
    auto wait_ahead = [&](int stages) {  // at most `stages` younger stages may stay in flight
      if constexpr (W_ROLE) {
        if (stages >= 6) wait_newer<6 * kLoadsW>();
        else if (stages == 5) wait_newer<5 * kLoadsW>();
        else if (stages == 4) wait_newer<4 * kLoadsW>();
        else if (stages == 3) wait_newer<3 * kLoadsW>();
        else if (stages == 2) wait_newer<2 * kLoadsW>();
        else if (stages == 1) wait_newer<kLoadsW>();
        else wait_newer<0>();
      } else {
        if (stages >= 2) wait_newer<2 * kLoadsH>();
        else if (stages == 1) wait_newer<kLoadsH>();
        else wait_newer<0>();
      }
    };

    const int npro = min(LEAD, T);
    for (int s = 0; s < npro; ++s) {
#pragma unroll
      for (int n = 0; n < NL; ++n) issue_one(n);
      loaded_step();
    }
    wait_ahead(npro - 1);  // own loads of stage 0 have landed
    lds_barrier();
    Frag f0, f1;
    read_frag(0, 0, f0);
    int sw = 0, sh = 0;               // stages of the current step in the two rings
    int tile_c = blockIdx.x, kc = 0;  // compute cursor
    auto next_stage = [&]() {
      sw = (sw + 1) & (kRingW - 1);
      sh = (sh + 1) & (kRingH - 1);
    };
    auto end_of_step = [&]() {  // tile finished: epilogue from the registers, next tile starts at zero
      if (++kc == nk) {
        store_logits_and_partials<2, CE>(a, acc, wm * 64, tile_c * SN + wn * 64, M, lane);
        clear_acc();
        kc = 0;
        tile_c += G;
      }
    };
    // Steady-state step t (t + LEAD < T): on entry `cur` holds the fragments of stage t.
    // Outstanding loads of this wavefront: stages t+1 .. t+LEAD-1 (and possibly the stores of an
    // epilogue, younger than all of them); it waits for its own loads of stage t+1, the barrier
    // publishes that stage and tells that everybody has left stage t-1, which is refilled with
    // step t+LEAD between the multiplies.  The fragment reads of the next stage sit in the middle
    // of the multiplies.
    auto step_steady = [&](const Frag& cur, Frag& nxt) {
      __builtin_amdgcn_sched_barrier(0);
      wait_newer<(LEAD - 2) * NL>();
      lds_barrier();
      next_stage();
      mfma_row(cur, 0, 0);
      issue_one(0);
      mfma_row(cur, 0, 1);
      issue_one(1);
      __builtin_amdgcn_sched_barrier(0);
      read_frag(sw, sh, nxt);
      __builtin_amdgcn_sched_barrier(0);
      mfma_row(cur, 1, 0);
      if constexpr (NL > 2) issue_one(2);
      mfma_row(cur, 1, 1);
      if constexpr (NL > 3) issue_one(3);
      __builtin_amdgcn_sched_barrier(0);
      loaded_step();
      end_of_step();
    };
    // General step for the end of the sequence: refills only while steps are left, waits by count.
    auto step_tail = [&](int t, const Frag& cur, Frag& nxt) {
      wait_ahead(min(t + LEAD - 1, T - 1) - t - 1);
      lds_barrier();
      next_stage();
      if (t + LEAD < T) {
#pragma unroll
        for (int n = 0; n < NL; ++n) issue_one(n);
        loaded_step();
      }
      if (t + 1 < T) read_frag(sw, sh, nxt);
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int i = 0; i < 2; ++i) mfma_row(cur, ks, i);
      end_of_step();
    };
    int t = 0;
    for (; t + kRingW < T; t += 2) {  // both steps refill in both roles: t + 1 + kRingW - 1 < T
      step_steady(f0, f1);
      step_steady(f1, f0);
    }
    for (; t < T; t += 2) {
      step_tail(t, f0, f1);
      step_tail(t + 1, f1, f0);
    }
  };
  if (wave < 4) run(std::integral_constant<int, 0>{});
  else run(std::integral_constant<int, 1>{});
}

}  // namespace

bool stream_supports(int M, int d) { return M <= SM && d % 64 == 0; }

hipError_t launch_head_stream(const HeadArgs& a) {
  const int n_tiles = (a.V + SN - 1) / SN;
  // one workgroup per CU (the kernel uses all of a CU's LDS); each walks its tiles back to back
  static int cus[64];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  if (cus[dev] == 0) {
    int n = 0;
    e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return e;
    cus[dev] = n > 0 ? n : 1;
  }
  const int grid = n_tiles < cus[dev] ? n_tiles : cus[dev];
  if (a.labels) FEF_LAUNCH_HEAD(head_stream_kernel<true>, dim3((unsigned)grid), dim3(512), a, a, n_tiles);
  else FEF_LAUNCH_HEAD(head_stream_kernel<false>, dim3((unsigned)grid), dim3(512), a, a, n_tiles);
  return hipGetLastError();
}

}  // namespace fef
