// Vocabulary-head kernel for 32 < M <= 128 rows through the head (a few sequences per call, or a
// DRAFT / TARGET call of up to 16 eight-token windows).  At these sizes the pass over W is still
// the cost (2 M V d flops need well under the time 1 GB of W takes from HBM), so the kernel is
// built around streaming W: one workgroup owns all M rows x 256 tokens and walks k in steps of
// 32.  W goes through a ring of eight 16 KB LDS stages filled by direct-to-LDS loads seven k-steps
// ahead (112 KB of W in flight per CU: with 64 bytes per row per step HBM latency under load is
// several microseconds, and five stages ahead left the loop waiting for data); H, which every
// workgroup re-reads and which therefore sits in L2, goes through a ring of four 8 KB stages three
// steps ahead.  Together they use the whole 160 KB of LDS.  The vector-memory counter of a
// wavefront completes in order, so two different leads cannot share a wavefront: wavefronts 0..3
// load W (four 1 KB loads per step each), wavefronts 4..7 load H (two per step each).
//
// Eight wavefronts as 2 (k halves of a 32-wide step) x 4 (64-token columns): each wavefront
// multiplies all 128 rows by its 64 tokens over its own 16-wide k-slice, 4 x 2
// v_mfma_f32_32x32x16_bf16 tiles (128 accumulator registers), so a k-step costs a wavefront six
// 16-byte fragment reads for eight multiplies.  The two k halves are added through LDS at the end
// (each wavefront keeps 64 of the 128 rows) in a fixed order, then the shared epilogue writes
// logits and (max, sum exp) partials.
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
  bf16x8 a[4], b[2];
};

template <bool CE>
__global__ __launch_bounds__(512) void head_stream128_kernel(HeadArgs a) {
  __shared__ bf16x8 ringW[kRingW * kStageW];  // 128 KB
  __shared__ bf16x8 ringH[kRingH * kStageH];  // 32 KB: one workgroup per CU
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kh = wave >> 2, wn = wave & 3;  // k half, token column
  const int j32 = lane & 31, h = lane >> 5;
  const int M = a.nrows;
  const int n0 = blockIdx.x * SN;

  floatx16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = floatx16{};

  // fragment read addresses inside a stage (chunks); the stage offset is added per step
  int fa[4], fb[2];
#pragma unroll
  for (int i = 0; i < 4; ++i) fa[i] = swz4(i * 32 + j32, kh * 2 + h);
#pragma unroll
  for (int j = 0; j < 2; ++j) fb[j] = swz4(wn * 64 + j * 32 + j32, kh * 2 + h);
  auto read_frag = [&](int sw, int sh, Frag& f) {
    const bf16x8* As = ringH + sh * kStageH;
    const bf16x8* Bs = ringW + sw * kStageW;
#pragma unroll
    for (int i = 0; i < 4; ++i) f.a[i] = As[fa[i]];
#pragma unroll
    for (int j = 0; j < 2; ++j) f.b[j] = Bs[fb[j]];
  };
  auto mfma_pair = [&](const Frag& f, int i) {
#pragma unroll
    for (int j = 0; j < 2; ++j)
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[i], f.b[j], acc[i][j], 0, 0, 0);
  };

  const int nk = a.d / SK;

  // The k loop for one loading role.  ROLE 0: this wavefront loads W rows [64 w, 64 w + 64) of
  // every stage (lead kRingW - 1); ROLE 1: H rows [32 (w - 4), +32) (lead kRingH - 1).  Lane l of
  // a load owns LDS slot (row + l/4, position l%4) and fetches the chunk the swizzle assigns to
  // that slot.  Rows past M / V re-read the last row; they are masked in the epilogue.
  auto k_loop = [&](auto role) {
    constexpr bool W_ROLE = decltype(role)::value == 0;
    constexpr int NL = W_ROLE ? kLoadsW : kLoadsH;     // loads per stage
    constexpr int LEAD = (W_ROLE ? kRingW : kRingH) - 1;
    constexpr int RING = LEAD + 1;
    const __bf16* gp[NL];
    uint32_t slot0[NL];  // LDS byte offset of load n in stage 0
#pragma unroll
    for (int n = 0; n < NL; ++n) {
      const int r = (W_ROLE ? wave * 64 : (wave - 4) * 32) + n * 16 + (lane >> 2);
      const int c = (lane & 3) ^ ((r >> 2) & 3);
      gp[n] = W_ROLE ? (const __bf16*)a.W + (size_t)min(n0 + r, a.V - 1) * a.d + c * 8
                     : h_row(a, min(r, M - 1)) + c * 8;
      const bf16x8* base = W_ROLE ? ringW : ringH;
      slot0[n] = lds_offset(base + ((W_ROLE ? wave * 64 : (wave - 4) * 32) + n * 16) * 4);
    }
    constexpr uint32_t kStageBytes = (W_ROLE ? kStageW : kStageH) * 16;
    // gp[] always point at the next k-step to be loaded, which goes to stage `s_load`
    int s_load = 0;
    auto issue_one = [&](int n) { load_to_lds_16(gp[n], slot0[n] + s_load * kStageBytes); gp[n] += SK; };
    auto advance_load = [&]() { s_load = s_load + 1 == RING ? 0 : s_load + 1; };

    const int npro = min(LEAD, nk);
    for (int s = 0; s < npro; ++s) {
#pragma unroll
      for (int n = 0; n < NL; ++n) issue_one(n);
      advance_load();
    }
    // wait for the own loads of stage 0: everything but the npro - 1 younger stages
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
    wait_ahead(npro - 1);
    lds_barrier();
    Frag f0, f1;
    read_frag(0, 0, f0);
    int sw = 0, sh = 0;  // stages of k-step kt in the two rings
    auto next_stage = [&]() {
      sw = (sw + 1) & (kRingW - 1);
      sh = (sh + 1) & (kRingH - 1);
    };
    // Steady-state k-step (kt + kRingW - 1 < nk): on entry `cur` holds the fragments of stage kt.
    // Outstanding loads of this wavefront: stages kt+1 .. kt+LEAD-1; it waits for its own loads of
    // stage kt+1, the barrier publishes that stage and tells that everybody has left stage kt-1,
    // which is refilled with k-step kt+LEAD between the multiplies.  One basic block; the
    // fragment reads of the next stage sit in the middle of the multiplies.
    auto step_steady = [&](const Frag& cur, Frag& nxt) {
      __builtin_amdgcn_sched_barrier(0);
      wait_newer<(LEAD - 2) * NL>();
      lds_barrier();
      next_stage();
      mfma_pair(cur, 0);
      issue_one(0);
      mfma_pair(cur, 1);
      issue_one(1);
      __builtin_amdgcn_sched_barrier(0);
      read_frag(sw, sh, nxt);
      __builtin_amdgcn_sched_barrier(0);
      mfma_pair(cur, 2);
      if constexpr (NL > 2) issue_one(2);
      mfma_pair(cur, 3);
      if constexpr (NL > 3) issue_one(3);
      advance_load();
    };
    // General k-step for the end of the loop: refills only while k-steps are left, waits by count.
    auto step_tail = [&](int kt, const Frag& cur, Frag& nxt) {
      wait_ahead(min(kt + LEAD - 1, nk - 1) - kt - 1);
      lds_barrier();
      next_stage();
      if (kt + LEAD < nk) {
#pragma unroll
        for (int n = 0; n < NL; ++n) issue_one(n);
        advance_load();
      }
      if (kt + 1 < nk) read_frag(sw, sh, nxt);
#pragma unroll
      for (int i = 0; i < 4; ++i) mfma_pair(cur, i);
    };
    int kt = 0;
    for (; kt + kRingW < nk; kt += 2) {  // both steps refill in both roles: kt + 1 + kRingW - 1 < nk
      step_steady(f0, f1);
      step_steady(f1, f0);
    }
    for (; kt < nk; kt += 2) {  // nk is even (d is a multiple of 64)
      step_tail(kt, f0, f1);
      step_tail(kt + 1, f1, f0);
    }
  };
  if (wave < 4) k_loop(std::integral_constant<int, 0>{});
  else k_loop(std::integral_constant<int, 1>{});
  lds_barrier();  // every load has landed and every fragment read is done: the rings are free

  // Add the two k halves.  A wavefront keeps two of its four row tiles (k half 0: rows 0..63,
  // k half 1: rows 64..127) and hands the other two to its partner (wave ^ 4) through LDS:
  // [wavefront][register 0..63][lane], conflict-free.  low + high in that order on both sides.
  float* ex = reinterpret_cast<float*>(ringW);
  floatx16 keep[2][2];
  {
    float* mine = ex + wave * (64 * 64);
    const float* theirs = ex + (wave ^ 4) * (64 * 64);
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float give = kh == 0 ? acc[2 + t][j][r] : acc[t][j][r];
          mine[((t * 2 + j) * 16 + r) * 64 + lane] = give;
        }
    lds_barrier();
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float got = theirs[((t * 2 + j) * 16 + r) * 64 + lane];
          keep[t][j][r] = kh == 0 ? acc[t][j][r] + got : got + acc[2 + t][j][r];
        }
  }
  store_logits_and_partials<2, CE>(a, keep, kh * 64, n0 + wn * 64, M, lane);
}

}  // namespace

bool stream128_supports(int M, int d) { return M <= SM && d % 64 == 0; }

hipError_t launch_head_stream128(const HeadArgs& a) {
  const int n_tiles = (a.V + SN - 1) / SN;
  if (a.labels) FEF_LAUNCH_HEAD(head_stream128_kernel<true>, dim3((unsigned)n_tiles), dim3(512), a, a);
  else FEF_LAUNCH_HEAD(head_stream128_kernel<false>, dim3((unsigned)n_tiles), dim3(512), a, a);
  return hipGetLastError();
}

}  // namespace fef
