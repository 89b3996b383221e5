// Vocabulary-head kernel for 32 < M <= 128 rows through the head (a few sequences per call, or a
// DRAFT / TARGET call of up to 16 eight-token windows).  At these sizes the pass over W is still
// the cost (2 M V d flops need well under the time 1 GB of W takes from HBM), so the kernel is
// built around streaming W without a pause.
//
// One persistent workgroup per CU takes an equal share of the vocabulary as 256-token tiles and walks k in steps of
// 32 over all of them as ONE sequence of steps: W goes through a ring of seven (eight with 64-row tiles) 16 KB LDS
// stages filled by direct-to-LDS loads six (seven) steps ahead (measured: a lead of three steps does as well;
// a wavefront with more loads outstanding than the memory pipeline takes blocks at its next load
// instruction, and that, not a wait for data, is where the loading wavefronts spend a third of
// their time), H, which every workgroup re-reads and which therefore sits in L2, through a ring
// of four 8 KB stages three steps ahead.  With 4 KB for the partials of a finished tile that is
// 148 of the 160 KB of LDS.  The loads run on across tile boundaries, so only the first
// tile of a workgroup pays the cold start, and the epilogue of a tile (registers, and 4 KB of LDS of its own)
// runs while the first stages of the next tile arrive.  The vector-memory counter of a wavefront
// completes in order, so two different leads cannot share a wavefront: wavefronts 0..3 load W
// (four 1 KB loads per step each), wavefronts 4..7 load H (two per step each).  The stores of an
// epilogue enter the same counter behind the loads in flight; the waits that follow are by count
// of the youngest operations, so they can only wait for more than they need, never for less.
//
// Eight wavefronts as 2 (row halves) x 4 (64-token columns), each NI x 2
// v_mfma_f32_32x32x16_bf16 tiles over the full k (NI = 2: 128 rows per tile, eight 16-byte
// fragment reads for eight multiplies per step; NI = 1 for M <= 64: 64 rows, half the multiplies,
// which at these sizes is less heat rather than less time: the kernel runs against the power
// limit, and the memory system slows down with the clocks), and a tile ends in the shared
// epilogue with no exchange between wavefronts.
//
// Each workgroup starts its walk over k at another k-step and wraps round.  Every row of W
// starts at a multiple of 2 d bytes, so workgroups that walk k in step ask HBM for the same low
// address bits at the same time and crowd the same channels; a plain read kernel with this
// access pattern gets 4.5 TB/s in step and 5.4 to 6.3 TB/s with staggered starts.
//
// LDS stages are [rows][4 chunks of 16 B], chunks swizzled as in the 256 x 256 kernel.
#include <type_traits>

#include "head_common.hpp"

namespace fef {
namespace {

constexpr int SM = 128, SN = 256, SK = 32;     // SM: rows of the largest tile
constexpr int kRingH = 4;                      // stages; loads run kRing - 1 k-steps ahead
constexpr int kStageW = SN * 4;                // 16-byte chunks per W stage
constexpr int kLoadsW = 4;                     // load instructions per W-loading wavefront per stage

template <int NI>
struct Frag {
  bf16x8 a[2][NI], b[2][2];  // [16-wide k-slice][32-row / 32-token tile]
};

// NI = 32-row tiles per wavefront: the workgroup tile has 64 NI rows.
template <int NI, bool CE>
__global__ __launch_bounds__(512) void head_stream_kernel(HeadArgs a_in, int n_units) {
  constexpr int kLoadsH = NI;                 // 16 rows per load, 16 NI rows per H-loading wavefront
  // 64-row tiles leave room for an eighth W stage (8 x 16 + 4 x 4 + 4 = 148 KB; 128-row tiles: 7 x 16 + 4 x 8 + 4),
  // and with it the head is 6 us faster at M = 64 than with seven
  constexpr int kRingW = NI == 1 ? 8 : 7;
  constexpr int kStageH = 64 * NI * 4;        // 16-byte chunks per H stage
  __shared__ bf16x8 ringW[kRingW * kStageW];
  __shared__ bf16x8 ringH[kRingH * kStageH];  // one workgroup per CU
  __shared__ float2 lpart[SM * 4];            // 4 KB: the four 64-token partials of each row of a tile, to be merged
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 2, wn = wave & 3;  // row half, token column
  const int j32 = lane & 31, h = lane >> 5;
  const int M = a_in.nrows;
  // This workgroup's tokens: units [u0, u1) of 64 tokens, an equal share of the vocabulary (a share of whole
  // 256-token tiles leaves the 594 tiles of a 151936-token vocabulary as three tiles for 82 workgroups and two for
  // the rest, and everybody waits for the 82; the kernel's time goes with the bytes a workgroup reads, and a last
  // tile of one to three 64-token columns reads that much less of W).  To the kernel the vocabulary ends where
  // the share ends: rows of W past it re-read the share's last row and are masked in the epilogue.
  const int G = gridDim.x;
  const int u0 = (int)((long)blockIdx.x * n_units / G), u1 = (int)((long)(blockIdx.x + 1) * n_units / G);
  HeadArgs a = a_in;
  a.V = min(a_in.V, u1 * 64);
  const int nk = a.d / SK;
  const int my_tiles = (u1 - u0 + 3) / 4;
  const int T = my_tiles * nk;  // steps of this workgroup; even, because nk is

  floatx16 acc[NI][2];
  auto clear_acc = [&]() {
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) acc[i][j] = floatx16{};
  };
  clear_acc();

  // fragment read addresses inside a stage (chunks); the stage offset is added per step
  int fa[2][NI], fb[2][2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
    for (int i = 0; i < NI; ++i) fa[ks][i] = swz4(wm * (32 * NI) + i * 32 + j32, ks * 2 + h);
#pragma unroll
    for (int j = 0; j < 2; ++j) fb[ks][j] = swz4(wn * 64 + j * 32 + j32, ks * 2 + h);
  }
  auto read_frag = [&](int sw, int sh, Frag<NI>& f) {
    const bf16x8* As = ringH + sh * kStageH;
    const bf16x8* Bs = ringW + sw * kStageW;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
      for (int i = 0; i < NI; ++i) f.a[ks][i] = As[fa[ks][i]];
#pragma unroll
      for (int j = 0; j < 2; ++j) f.b[ks][j] = Bs[fb[ks][j]];
    }
  };
  // fragment r of a stage, in the order the multiplies use them: slice 0 (a.., b0, b1), then slice 1
  auto read_one = [&](int sw, int sh, Frag<NI>& f, int r) {
    const bf16x8* As = ringH + sh * kStageH;
    const bf16x8* Bs = ringW + sw * kStageW;
    const int ks = r / (NI + 2), q = r % (NI + 2);
    if (q < NI) f.a[ks][q] = As[fa[ks][q]];
    else f.b[ks][q - NI] = Bs[fb[ks][q - NI]];
  };
  // The multiplies of one k-slice in two parts: row tile `part` when NI = 2, token tile `part` when NI = 1.
  auto mfma_part = [&](const Frag<NI>& f, int ks, int part) {
    if constexpr (NI == 1) {
      acc[0][part] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[ks][0], f.b[ks][part], acc[0][part], 0, 0, 0);
    } else {
#pragma unroll
      for (int j = 0; j < 2; ++j)
        acc[part][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[ks][part], f.b[ks][j], acc[part][j], 0, 0, 0);
    }
  };

  // The whole sequence of steps for one loading role.  ROLE 0: this wavefront loads W rows
  // [64 w, 64 w + 64) of every stage (lead kRingW - 1); ROLE 1: H rows [16 NI (w - 4), + 16 NI)
  // (lead kRingH - 1).  Lane l of a load owns LDS slot (row + l/4, position l%4) and fetches the chunk
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
      const int r0 = (W_ROLE ? wave * 64 : (wave - 4) * (16 * NI)) + n * 16;
      lrow[n] = r0 + (lane >> 2);
      lchunk[n] = ((lane & 3) ^ ((lrow[n] >> 2) & 3)) * 8;
      slot0[n] = lds_offset((W_ROLE ? ringW : ringH) + r0 * 4);
    }
    // This workgroup's walk over k starts at k-step k0 and wraps round: step t of a tile is
    // k-step (k0 + t) mod nk, in both roles.
    const int k0 = (int)((blockIdx.x * 37u) % (unsigned)nk);
    // loader cursor: the next step to load is k-step kl of tile tile_l and goes to stage s_load
    int tile_l = 0, kl = 0, s_load = 0, t_load = 0;  // tiles count from the share's first token
    auto retarget = [&]() {  // gp[] at the first k-step of tile tile_l
#pragma unroll
      for (int n = 0; n < NL; ++n)
        gp[n] = (W_ROLE ? (const __bf16*)a.W + (size_t)min(u0 * 64 + tile_l * SN + lrow[n], a.V - 1) * a.d
                        : h_row(a, min(lrow[n], M - 1))) + lchunk[n] + k0 * SK;
    };
    retarget();
    auto issue_one = [&](int n) {
      load_to_lds_16(gp[n], __builtin_amdgcn_readfirstlane(slot0[n] + s_load * kStageBytes));
      gp[n] += SK;
    };
    // All NL loads of a step behind one write of M0: load n lands 1024 n bytes further on in LDS, and the
    // instruction offset moves the memory address by as much, which the operand takes back.  A write of
    // M0 in front of every load holds the wavefront (and its multiplies) for some tens of cycles each:
    // one per step instead of four is worth 2.3 % at M = 128 and 3.5 % at M = 64.
    auto issue_all = [&]() {
      const uint32_t base = __builtin_amdgcn_readfirstlane(slot0[0] + s_load * kStageBytes);
      if constexpr (NL == 4)
        asm volatile("s_mov_b32 m0, %4\n\ts_nop 0\n\t"
                     "global_load_lds_dwordx4 %0, off\n\tglobal_load_lds_dwordx4 %1, off offset:1024\n\t"
                     "global_load_lds_dwordx4 %2, off offset:2048\n\tglobal_load_lds_dwordx4 %3, off offset:3072"
                     :: "v"(gp[0]), "v"(gp[1] - 512), "v"(gp[2] - 1024), "v"(gp[3] - 1536), "s"(base) : "memory");
      else if constexpr (NL == 2)
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\t"
                     "global_load_lds_dwordx4 %0, off\n\tglobal_load_lds_dwordx4 %1, off offset:1024"
                     :: "v"(gp[0]), "v"(gp[1] - 512), "s"(base) : "memory");
      else
        load_to_lds_16(gp[0], base);
#pragma unroll
      for (int n = 0; n < NL; ++n) gp[n] += SK;
    };
    auto loaded_step = [&]() {  // bookkeeping after the NL loads of one step
      s_load = s_load + 1 == RING ? 0 : s_load + 1;
      ++t_load;
      if (++kl == nk) {
        kl = 0;
        tile_l += 1;
        if (t_load < T) retarget();
      } else if (kl == nk - k0) {  // back to k = 0
#pragma unroll
        for (int n = 0; n < NL; ++n) gp[n] -= a.d;
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
    Frag<NI> f0, f1;
    read_frag(0, 0, f0);
    int sw = 0, sh = 0;               // stages of the current step in the two rings
    int tile_c = 0, kc = 0;  // compute cursor
    float run_mx = -INFINITY, run_sum = 0.f;  // thread tid < 64 NI: (max, sum exp) of row tid over the tiles done so far
    auto next_stage = [&]() {
      sw = sw + 1 == kRingW ? 0 : sw + 1;
      sh = (sh + 1) & (kRingH - 1);
    };
    // Tile finished: epilogue from the registers, next tile starts at zero.  The four 64-token partials of a row
    // (one per wavefront column) meet in LDS, where the thread that owns the row folds them into its running
    // partial; the workgroup leaves ONE partial per row, over all its tokens, at the end: 256 partials per row for
    // the kernels that follow.  Every wavefront, whatever it loads, finishes its tiles at the same steps, so the
    // barrier is met by all; the next tile's partials are written at least two step barriers later.
    auto end_of_step = [&]() {
      if (++kc == nk) {
        store_logits_and_partials<NI, CE, 8>(a, acc, wm * (32 * NI), u0 * 64 + tile_c * SN + wn * 64, M, lane, lpart,
                                             wm * (32 * NI), wn);
        lds_barrier();
        if (tid < 64 * NI && tid < M) {
          constexpr float kLog2e = 1.4426950408889634f;
          float2 p[4];
#pragma unroll
          for (int c = 0; c < 4; ++c) p[c] = lpart[tid * 4 + c];
          const float mx = fmaxf(fmaxf(run_mx, p[0].x), fmaxf(fmaxf(p[1].x, p[2].x), p[3].x));  // finite: the tile's first token exists
          float sum = run_sum * exp2f((run_mx - mx) * kLog2e);
#pragma unroll
          for (int c = 0; c < 4; ++c) sum += p[c].y * exp2f((p[c].x - mx) * kLog2e);
          run_mx = mx;
          run_sum = sum;
        }
        clear_acc();
        kc = 0;
        tile_c += 1;
      }
    };
    // Steady-state step t (t + LEAD < T): on entry `cur` holds the fragments of stage t.
    // Outstanding loads of this wavefront: stages t+1 .. t+LEAD-1 (and possibly the stores of an
    // epilogue, younger than all of them); it waits for its own loads of stage t+1, the barrier
    // publishes that stage and tells that everybody has left stage t-1, which is refilled with
    // step t+LEAD between the multiplies.  The fragment reads of the next stage sit in the middle
    // of the multiplies.
    auto step_steady = [&](const Frag<NI>& cur, Frag<NI>& nxt) {
      __builtin_amdgcn_sched_barrier(0);
      wait_newer<(LEAD - 2) * NL>();
      lds_barrier();
      next_stage();
      if constexpr (NI == 2) {
        // 128-row tiles: the eight multiplies of the step in order, one fragment read of the next stage after each
        // (in the order the next step uses them), the loads after the second: -2 % against reading the eight
        // fragments in one run.  (With 64-row tiles, four multiplies and six reads per step, the run is faster.)
#pragma unroll
        for (int n = 0; n < 8; ++n) {
          const int ks = n >> 2, i = (n >> 1) & 1, j = n & 1;
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur.a[ks][i], cur.b[ks][j], acc[i][j], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
          read_one(sw, sh, nxt, n);
          __builtin_amdgcn_sched_barrier(0);
          if (n == 1) {
            issue_all();
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      } else {
        mfma_part(cur, 0, 0);
        issue_all();
        mfma_part(cur, 0, 1);
        __builtin_amdgcn_sched_barrier(0);
        read_frag(sw, sh, nxt);
        __builtin_amdgcn_sched_barrier(0);
        mfma_part(cur, 1, 0);
        mfma_part(cur, 1, 1);
        __builtin_amdgcn_sched_barrier(0);
      }
      loaded_step();
      end_of_step();
    };
    // General step for the end of the sequence: refills only while steps are left, waits by count.
    auto step_tail = [&](int t, const Frag<NI>& cur, Frag<NI>& nxt) {
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
        for (int part = 0; part < 2; ++part) mfma_part(cur, ks, part);
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
    if (tid < 64 * NI && tid < M) a.partials[(size_t)tid * a.nT + blockIdx.x] = make_float2(run_mx, run_sum);
  };
  if (wave < 4) run(std::integral_constant<int, 0>{});
  else run(std::integral_constant<int, 1>{});
}

}  // namespace

bool stream_supports(int M, int d) { return M <= SM && d % 64 == 0; }

// One workgroup per CU of a 256-CU device (the kernel uses most of a CU's LDS), fewer when the vocabulary has fewer
// than 256 tiles of 256 tokens; workgroup b takes units floor(b U / G) .. floor((b + 1) U / G) of 64 tokens.
int stream_grid(int V) {
  const int units = (V + 63) / 64, want = (units + 3) / 4;
  return want < kSkinnyMaxGrid ? want : kSkinnyMaxGrid;
}

template <int NI>
static void launch_stream(const HeadArgs& a, int grid, int n_units) {
  if (a.labels) FEF_LAUNCH_HEAD((head_stream_kernel<NI, true>), dim3((unsigned)grid), dim3(512), a, a, n_units);
  else FEF_LAUNCH_HEAD((head_stream_kernel<NI, false>), dim3((unsigned)grid), dim3(512), a, a, n_units);
}

hipError_t launch_head_stream(const HeadArgs& a) {
  const int n_units = (a.V + 63) / 64, grid = stream_grid(a.V);
  if (a.nrows <= 64) launch_stream<1>(a, grid, n_units);
  else launch_stream<2>(a, grid, n_units);
  return hipGetLastError();
}

}  // namespace fef
