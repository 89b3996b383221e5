// Shared declarations of the verify-step library: kernel launchers, the Philox generator
// and wavefront / workgroup scan primitives.  gfx950 only (64-wide wavefronts).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fef {

constexpr int kWave = 64;
constexpr int kMaxBlock = 4096;  // positions per block (FEF_MAX_BLOCK)
constexpr int kMaxK = 64;        // window (FEF_MAX_K): one ballot covers a window

// ---------------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11).  key = (seed lo, seed hi); counter = (position, step,
// sequence, stream); word 0 of the output is used.
// ---------------------------------------------------------------------------------------------
constexpr uint32_t kStreamDraft = 0, kStreamAccept = 1, kStreamResidual = 2, kStreamRecorrupt = 3;

__host__ __device__ inline uint32_t philox_word0(uint64_t seed, uint32_t c0, uint32_t c1,
                                                 uint32_t c2, uint32_t c3) {
  uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    if (r) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    c1 = (uint32_t)p1; c3 = (uint32_t)p0; c0 = n0; c2 = n2;
  }
  return c0;
}

// Top 23 bits -> u = (n + 1/2) 2^-23 in (0,1); every value is exact in fp32.
__host__ __device__ inline float word_to_uniform(uint32_t w) {
  return ((float)(w >> 9) + 0.5f) * 1.1920928955078125e-07f;
}

__host__ __device__ inline float philox_uniform(uint64_t seed, uint32_t position, uint32_t step,
                                                uint32_t sequence, uint32_t stream) {
  return word_to_uniform(philox_word0(seed, position, step, sequence, stream));
}

// ---------------------------------------------------------------------------------------------
// Arguments of the vocabulary-head kernels: L[r, v] = inv_tau * sum_k H[r, k] W[v, k] for the
// 2*BK rows (draft rows first), written once as fp32, plus per (row, vocab tile of `tn`)
// partials (max, sum exp(L - max)) for the log-sum-exp.
// ---------------------------------------------------------------------------------------------
struct HeadArgs {
  const void* h_draft;   // [BK, d]
  const void* h_target;  // [BK, d]
  const void* W;         // [V, d]
  int BK, d, V;
  int row0, nrows;       // rows [row0, row0 + nrows) of the stacked [draft; target] matrix
  float inv_tau;
  float* logits;         // [nrows, ldl]: already points at row row0
  long ldl;
  float2* partials;      // [nrows, nT]: already points at row row0
  int nT;                // partial tiles per row
  // Cross-entropy use of the head (labels != NULL): no logits are written (logits == NULL) and
  // the scaled logit of each row's label token goes to label_logit[row].
  const int32_t* labels;  // [nrows] token id per row, negative = row does not count
  float* label_logit;     // [nrows]
  hipStream_t stream;
  hipEvent_t ev_begin, ev_end;  // optional: receive the kernel's own start / stop timestamps
};

constexpr int kSkinnyUnit = 16;     // the skinny kernel walks W in tiles of 16 tokens ...
constexpr int kSkinnyMaxGrid = 256;  // ... split evenly over at most one workgroup per CU, and
                                     // writes one partial per (row, workgroup)
constexpr int kTiledTn = 64;         // partial-tile width of the tiled and f32 kernels, share unit of the LDS-streaming kernel
constexpr int kTiled256Tn = 256;     // ... of the 256 x 256 kernels (merged through LDS in their epilogue)

bool skinny_supports(int M, int d);
hipError_t launch_head_skinny(const HeadArgs& a);
hipError_t launch_head_tiled(const HeadArgs& a);
hipError_t launch_head_tiled256(const HeadArgs& a);
bool stream_supports(int M, int d);
int stream_grid(int V);     // workgroups = partial slots per row
hipError_t launch_head_stream(const HeadArgs& a);
bool rowstream_supports(int M, int d);
int rowstream_grid(int V);  // workgroups = partial slots per row
hipError_t launch_head_rowstream(const HeadArgs& a);
hipError_t launch_head_f32(const HeadArgs& a);

// ---------------------------------------------------------------------------------------------
// Arguments of the sampling / verification kernels that follow the head.
// ---------------------------------------------------------------------------------------------
constexpr int kResidChunk = 256;  // vocabulary entries per residual-mass chunk

struct SeqState {
  int window, acc_len;
  float rej_lse_q, rej_lse_p;  // log-sum-exps of the rejected slot's draft / target row (if acc_len < window)
  int rej_pos, rej_xtarget;    // its block offset; greedy variant: the arg max of its target row
  int x[kMaxK];       // draft tokens of the window
  float ptok[kMaxK];  // pi(x~)
};

struct VerifyArgs {
  int B, K, block, V;
  int row0, nrows;          // logits rows the LSE / draft kernel handles in this call
  int phase;                // 0 fused, 1 draft half only, 2 target half only, 3 baseline top-n step
  long ldl;
  const float* logits;      // [2*B*K, ldl]
  const float2* partials;   // [2*B*K, nT]
  int nT;                   // partial tiles per row
  int tile_unit, tile_T, tile_G;  // tile i covers tokens [unit*floor(i*T/G), unit*floor((i+1)*T/G))
  uint64_t seed;
  uint32_t step, seq_base, pos_base;
  int n_rm, final_pass, lowconf_scope;
  float recorrupt_prob;
  int greedy;
  int n_transfer;            // baseline step only: positions committed per step
  const uint8_t* mask_in;
  uint8_t* pass_mask;
  float* conf;
  const int32_t* draft_tokens_in;
  int n_pass;                // with seq_pass: number of generation passes
  int32_t* seq_pass;         // [B] optional per-sequence pass counter (replaces final_pass)
  int32_t* seq_rounds;       // [B] optional round counter
  int32_t* tokens_state;     // [B, block] optional token state of the block
  // workspace
  float* lse;               // [2*B*K]
  int32_t* xdraft;          // [B*K]
  int32_t* xtarget;         // [B*K] greedy variant: arg max of the target rows
  int32_t* slot_pos;        // [B*K]
  int32_t* window;          // [B]
  struct SeqState* seqstate;  // [B] accept-phase results handed to the final kernel
  float* rmass;             // [nslots, nRC] residual mass per chunk
  float* amass;             // [nslots, nRC] overlap mass per chunk (all_slots only)
  int nRC;                  // ceil(V / kResidChunk)
  int all_slots;            // 1: masses for every slot (diagnostics), 0: rejected slot only
  // outputs
  int32_t* out_tokens; int32_t* out_accept_len; uint8_t* out_remask;
  int32_t* diag_draft_tokens; float* diag_alpha; float* diag_resid_mass; float* diag_lse;
  float* diag_logits; float* diag_conf_tok;
  hipStream_t stream;
};

hipError_t launch_verify(const VerifyArgs& a);

// Cross-entropy finish: per-row log-sum-exp from the partials, ce = lse - label logit, then the
// sum over rows in a fixed order.
struct CeArgs {
  int R, nT;
  const float2* partials;   // [R, nT]
  const int32_t* labels;    // [R]
  const float* label_logit; // [R]
  float* out_ce;            // [R]
  float* out_loss;          // [1]
  hipStream_t stream;
};
hipError_t launch_ce_init(float* label_logit, int R, hipStream_t stream);
hipError_t launch_ce_finish(const CeArgs& a);

}  // namespace fef
