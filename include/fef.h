/* fef.h - C ABI of the FeF-DLLM speculative verify step for AMD Instinct MI355X (gfx950).
 *
 * One call = one speculative round of the paper's full-sequence decoding algorithm
 * (Algorithm 2, body of the while-loop) for B independent sequences, followed by the
 * low-confidence re-corruption of the same algorithm when the round resolves the block:
 *
 *   window      b = min{k, L}: the first k unresolved positions of the block, ascending
 *   draft laws  rho^{j_m} = softmax(h_draft[m]  W^T / tau)
 *   draft       x~^{j_m} ~ rho^{j_m}                        (inverse CDF, ascending token id)
 *   target laws pi^{j_m}  = softmax(h_target[m] W^T / tau)
 *   accept      u_m <= min{1, pi(x~)/rho(x~)}, left to right, stop at the first failure
 *   correct     Z ~ [pi - rho]_+ / (1 - sum_z min{pi, rho})   (residual-distribution equation)
 *   commit      token and confidence c = pi(token) for accepted slots and the corrected one
 *   re-mask     if no unresolved position is left and this is not the final pass:
 *               the n_rm committed positions of the pass with the lowest confidence are
 *               re-corrupted through the absorbing forward kernel: each returns to the MASK
 *               state with probability recorrupt_prob (1 by default) and keeps its token
 *               otherwise (the re-corruption line of Algorithm 2, a draw from the forward
 *               kernel given the predicted clean token)
 *
 * The model forwards that produce the hidden states are outside the library.  The vocabulary
 * head W is shared by both laws (the paper instantiates draft and target with one network).
 *
 * All random draws come from Philox4x32-10, key = (seed low, seed high), counter =
 * (pos_base + block offset of the slot, step, seq_base + b, stream), output word 0,
 * stream 0 = draft sample, 1 = accept test, 2 = residual sample, 3 = re-corruption of a
 * selected position (masked iff u < recorrupt_prob); a word w becomes
 * u = ((w >> 9) + 0.5) * 2^-23.  A call is therefore a pure function of its arguments.
 * (The greedy variant, fef_params.greedy, replaces the three token draws by arg maxes.)
 *
 * Conventions
 *   - Plain C.  Every data pointer below is a DEVICE pointer owned by the caller unless it
 *     says "host".  fef_params itself lives in host memory.
 *   - The library allocates nothing: scratch space is the caller's `workspace`
 *     (fef_workspace_bytes tells how much; fef_verify_step_static uses a buffer built into the
 *     library instead).  No result depends on an earlier call; the only thing the library
 *     remembers is a per-device constant it looks up once (the address of the built-in buffer).
 *     The kernels' grids are sized for the 256 compute units of the device they are written for.
 *   - All work is enqueued on `stream`; the call returns without synchronising and the
 *     outputs are valid in stream order.  Concurrent calls need distinct workspaces.
 *   - Return value: FEF_OK or a negative fef_status.  Arguments are validated on the host
 *     before anything is launched; on error nothing is enqueued and nothing is written.
 *     fef_last_error() returns a thread-local description of the last failure.
 *   - Limits: 1 <= K <= min(block, FEF_MAX_K); block <= FEF_MAX_BLOCK; B, V >= 1;
 *     B*K <= 2^24; bf16: d a positive multiple of 64; f32: any d >= 1 and 2*B*K <= 65535.
 *     Row offsets are 64-bit, so 2*B*K*V may exceed 2^31.
 *     h_draft, h_target, W_vocab and workspace must be 16-byte aligned.
 */
#ifndef FEF_H
#define FEF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FEF_MAX_K 64
#define FEF_MAX_BLOCK 4096
#define FEF_ABI_VERSION 10
#define FEF_STATIC_SCRATCH_BYTES (32u << 20) /* built-in scratch of fef_verify_step_static        */

typedef enum {
  FEF_OK = 0,
  FEF_ERR_INVALID_ARG = -1, /* NULL / misaligned pointer, size or parameter out of range   */
  FEF_ERR_UNSUPPORTED = -2, /* valid request that no kernel here serves                    */
  FEF_ERR_WORKSPACE = -3,   /* workspace NULL or smaller than fef_workspace_bytes          */
  FEF_ERR_HIP = -4          /* a HIP runtime call failed (see fef_last_error)              */
} fef_status;

typedef enum {
  FEF_BF16 = 0, /* h_draft, h_target, W_vocab are bfloat16; MFMA path                      */
  FEF_F32 = 1   /* all three are float32; plain FMA path for tiny instances                */
} fef_dtype;

/* Which vocabulary-head kernel to run.  AUTO picks by (dtype, M, d), M = rows through the head
 * in this call: 2*B*K fused, B*K in a DRAFT or TARGET call. */
typedef enum {
  FEF_GEMM_AUTO = 0,
  FEF_GEMM_SKINNY = 1, /* bf16, M <= 32, d in {512, 1024, 2048, 2560, 3072, 3584, 4096}: W streamed
                          once, split-k; other d at M <= 32 go to STREAM (fef_select_gemm tells) */
  FEF_GEMM_TILED = 2,  /* bf16, any M: plain 128x128 LDS-tiled MFMA GEMM (never picked by AUTO) */
  FEF_GEMM_F32 = 3,    /* f32, any shape: reference-grade FMA kernel                       */
  FEF_GEMM_TILED256 = 4, /* bf16, any M: 256x256 LDS-tiled MFMA GEMM, eight wavefronts of 128x64 up to
                            256 rows, four of 128x128 above (AUTO: M > 128)                  */
  FEF_GEMM_STREAM = 5,   /* bf16, M <= 128: all rows x 256 tokens per persistent workgroup, W
                            streamed through a deep LDS ring, 64- or 128-row tiles (AUTO: 32 < M <= 128
                            where the other streaming kernel is not chosen)                  */
  FEF_GEMM_ROWSTREAM = 6 /* bf16, M <= 128, d a multiple of 512: every wavefront streams the W rows
                            of its own 16-token tiles into registers, H through LDS, 64-, 96- or
                            128-row tiles (AUTO: 32 < M <= 48 and 64 < M <= 96, where it needs
                            fewer rows than the kernel above)                                */
} fef_gemm_variant;

/* In Algorithm 2 the verification inputs X^(j_m) carry the draft prefix, so a real target
 * forward can only run after the draft tokens exist.  FUSED does both laws in one pass over W
 * (hidden states given up front).  DRAFT projects the draft rows only, samples x~ and writes
 * them to out_tokens (out_accept_len / out_remask are not touched and may be NULL; h_target is
 * not read and may be NULL).  TARGET projects the target rows only and finishes the round; it
 * must follow a DRAFT call with the same sizes, mask_in, seed, step and the SAME workspace,
 * left untouched in between (it holds the draft logits, their log-sum-exp and x~); h_draft is
 * not read and may be NULL.  DRAFT + TARGET give bit-identical results to FUSED when both
 * use the same head kernel, and read W twice.  The two calls may pass different W_vocab of the
 * same shape: a separate draft model with its own output embedding (the "A / B" rows of the
 * ablation on the choice of draft model). */
typedef enum { FEF_PHASE_FUSED = 0, FEF_PHASE_DRAFT = 1, FEF_PHASE_TARGET = 2 } fef_phase;

typedef struct {
  uint32_t struct_size;   /* = sizeof(fef_params); rejects callers built against another ABI */
  int32_t B;              /* sequences in this call                                          */
  int32_t d;              /* hidden size                                                     */
  int32_t V;              /* vocabulary size (every id in [0, V) is a valid token)           */
  int32_t dtype;          /* fef_dtype of h_draft, h_target, W_vocab                         */
  float temperature;      /* tau > 0; both laws are softmax(logits / tau)                    */
  uint32_t step;          /* index of this round; second Philox counter word                 */
  uint32_t seq_base;      /* global index of sequence 0; third Philox counter word is +b     */
  uint32_t pos_base;      /* absolute position of block offset 0; first counter word is +off */
  int32_t n_rm;           /* re-mask budget of LowConf; < 0 means block / 2                  */
  int32_t final_pass;     /* nonzero: last generation pass, no re-masking                    */
  int32_t lowconf_scope;  /* 0: candidates = positions committed in this pass (pass_mask);
                             1: every position of the block                                  */
  int32_t gemm_variant;   /* fef_gemm_variant                                                */
  const uint8_t* mask_in; /* [B, block] 1 = unresolved; NULL = whole block unresolved        */
  uint8_t* pass_mask;     /* [B, block] in/out: committed in the current pass; NULL = empty  */
  float* conf;            /* [B, block] in/out: confidence of resolved positions.  May be
                             NULL only if pass_mask is NULL and lowconf_scope == 0           */
  const int32_t* draft_tokens; /* [B, K] optional: verify these instead of sampling drafts   */
  /* optional diagnostic outputs, NULL = not wanted */
  int32_t* diag_draft_tokens;  /* [B, K] sampled (or given) draft tokens, -1 beyond window   */
  float* diag_alpha;           /* [B, K] sum_v min(p_v, q_v)                                 */
  float* diag_resid_mass;      /* [B, K] sum_v max(0, p_v - q_v)                             */
  float* diag_lse;             /* [2, B, K] log-sum-exp of draft / target logits             */
  float* diag_logits;          /* [2, B, K, V] scaled logits (draft rows first)              */
  float* diag_conf_tok;        /* [B, K] pi(committed token) per slot, 0 where none          */
  void* workspace;             /* device scratch, 256-byte aligned                           */
  size_t workspace_bytes;
  void* stream;                /* hipStream_t; NULL = the null stream                        */
  void* ev_head_begin;         /* optional hipEvent_t pair (both or neither) that receives    */
  void* ev_head_end;           /* the vocabulary-head kernel's own start / stop timestamps    */
  /* Optional device-side state of Algorithm 2's outer loops, so that a caller can enqueue the
   * rounds of a block back to back without reading anything back (all NULL = not used):       */
  int32_t n_pass;              /* N_step, the number of generation passes; >= 1 with seq_pass */
  int32_t* seq_pass;           /* [B] in/out: pass s of each sequence.  When given it replaces
                                  final_pass (a sequence is on its final pass iff s >= n_pass-1);
                                  s is incremented when LowConf fires and set to n_pass when the
                                  final pass resolves the block (the sequence is then done and
                                  further rounds leave it untouched)                           */
  int32_t* seq_rounds;         /* [B] in/out: incremented when the sequence had a non-empty
                                  window in this round                                        */
  int32_t* tokens_state;       /* [B, block] in/out: X restricted to the block; committed tokens
                                  are written at their positions, re-masked positions get -1   */
  int32_t phase;               /* fef_phase: the call order of the method when the target
                                  forward needs the draft tokens (see fef_phase)              */
  float recorrupt_prob;        /* in (0, 1]: probability 1 - alpha-bar_t with which a position
                                  selected by LowConf returns to MASK (absorbing forward kernel
                                  of Algorithm 2's re-corruption step); 1 = always.  With
                                  seq_pass, a selection that re-corrupts nothing leaves no
                                  unresolved position for any later pass: the sequence is
                                  marked done (s = n_pass)                                     */
  int32_t greedy;              /* 1: zero-temperature limit of the two laws.  Both become point
                                  masses at their arg max (lowest token id on a tie): x~ = arg max
                                  of the draft logits (or the given draft token), a slot is
                                  accepted iff x~ equals the arg max of the target logits, the
                                  corrected token is that arg max, and no uniform is drawn.
                                  Confidences stay softmax(logits / tau)(token).  0: sample      */
} fef_params;

/* Bytes of device workspace a call with these sizes needs (depends on B, d, V, dtype,
 * gemm_variant, K, block and on whether diag_alpha / diag_resid_mass are requested).
 * Returns 0 if the arguments are invalid. */
size_t fef_workspace_bytes(const fef_params* prm, int32_t K, int32_t block);

/* One speculative round.  Argument order follows the statement of the problem:
 *   h_draft   [B, K, d]  device, hidden state of window slot m in row m (draft forward)
 *   h_target  [B, K, d]  device, prefix-conditioned target hidden state of slot m
 *   W_vocab   [V, d]     device, row v = output embedding of token v (k contiguous)
 *   K                    speculative window k
 *   block                number of positions in the block
 *   seed                 Philox key
 *   out_tokens      [B, K]     device int32: committed token of slot m; -1 for slots after
 *                              the corrected one and beyond the window
 *   out_accept_len  [B]        device int32: accepted drafts a in [0, b]; committed
 *                              positions are min(a+1, b)
 *   out_remask      [B, block] device uint8: unresolved positions after the round
 * Rows of h_* for slots beyond a sequence's window are read but ignored. */
fef_status fef_verify_step(const fef_params* prm, const void* h_draft, const void* h_target,
                           const void* W_vocab, int32_t K, int32_t block, uint64_t seed,
                           int32_t* out_tokens, int32_t* out_accept_len, uint8_t* out_remask);

/* fef_verify_step for callers that cannot allocate device memory and have no workspace to hand
 * over: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, kernels and results as fef_verify_step (all three phases), except that
 * prm->workspace and prm->workspace_bytes are ignored: the scratch is a buffer of
 * FEF_STATIC_SCRATCH_BYTES (32 MiB) built into the library, one copy per GPU, held until the
 * process ends.  The call allocates nothing.  A call whose fef_workspace_bytes exceeds that size
 * (at V = 126464: more than 64 rows through the head, 2*B*K fused) returns FEF_ERR_WORKSPACE and
 * enqueues nothing.  The buffer keeps the previous call's contents; nothing in it has to start at
 * zero (every word is written before it is read within a call), and a TARGET call finds what the
 * DRAFT call before it left there.  All calls on one GPU share the buffer: calls that overlap in
 * time on one GPU (different streams or threads) race, so order them.  The first call on a device
 * looks the buffer's address up (with that device current); make it outside graph capture. */
fef_status fef_verify_step_static(const fef_params* prm, const void* h_draft, const void* h_target,
                                  const void* W_vocab, int32_t K, int32_t block, uint64_t seed,
                                  int32_t* out_tokens, int32_t* out_accept_len, uint8_t* out_remask);

/* The decoding step the paper's speed-ups are measured against (Main Results: LLaDA decodes one
 * token per step, the LLaDA/2 variant two): every window position gets its law from ONE forward,
 * p = softmax(h[m] W^T / tau); a token is drawn from it (inverse CDF with the draft stream's
 * uniform, or the arg max when prm->greedy) with confidence p(token); the n_transfer most
 * confident positions of the window are committed (equal confidences: the lower position first),
 * the others stay MASK.
 *   h             [B, K, d]  device: hidden state of window slot m in row m
 *   out_tokens    [B, K]     committed token of slot m, -1 where the slot was not committed
 *   out_committed [B]        min(n_transfer, window)
 *   out_remask    [B, block] unresolved positions after the step
 * Fields of prm that are read: as in a FEF_PHASE_DRAFT call (which fixes head kernel and workspace
 * size: fef_workspace_bytes with phase = DRAFT), plus greedy, conf and tokens_state (updated at
 * the committed positions), diag_draft_tokens (the drawn token of every slot), diag_conf_tok
 * (its confidence), diag_lse (first B*K entries), diag_logits.  prm->phase must be FUSED (0);
 * draft_tokens, pass_mask, seq_pass and seq_rounds must be NULL. */
fef_status fef_topn_step(const fef_params* prm, const void* h, const void* W_vocab, int32_t K, int32_t block,
                         uint64_t seed, int32_t n_transfer, int32_t* out_tokens, int32_t* out_committed,
                         uint8_t* out_remask);

/* The head kernel AUTO would choose for these sizes (a fef_gemm_variant), or a negative
 * fef_status.  Pure host function. */
int32_t fef_select_gemm(const fef_params* prm, int32_t K);

/* Training-side use of the same head (Algorithm 1, position-conditioned training, the
 * token-level loss CE_{j_m} = -log p_theta(X_0^{j_m} | X^(j_m), t) and its sum over the
 * prediction positions), forward only.  Row m of h is the predictor's hidden state at position
 * j_m for the position-conditioned input X^(j_m); p_theta = softmax(h_m W^T / tau).  The head
 * kernels run with their log-sum-exp epilogue and write no logits at all:
 *   h         [R, d]  device, dtype prm->dtype, 16-byte aligned
 *   W_vocab   [V, d]  device, same dtype
 *   labels    [R]     device int32: the clean token X_0^{j_m}, in [0, V); a negative value marks
 *                     a row that does not count (its CE is 0).  A value >= V gives CE = NaN.
 *   out_ce    [R]     device float: CE per row
 *   out_loss  [1]     device float: sum of out_ce in a fixed order; may be NULL
 * Fields of prm that are read: struct_size, d, V, dtype, temperature, gemm_variant (AUTO,
 * STREAM for R <= 128, TILED256, or F32 for f32 inputs), workspace, workspace_bytes (at least
 * fef_cross_entropy_workspace_bytes), stream, ev_head_begin / ev_head_end.  Same conventions and
 * error behaviour as fef_verify_step. */
size_t fef_cross_entropy_workspace_bytes(const fef_params* prm, int32_t R);
fef_status fef_head_cross_entropy(const fef_params* prm, const void* h, const void* W_vocab,
                                  const int32_t* labels, int32_t R, float* out_ce, float* out_loss);

/* Philox4x32-10 word 0 -> uniform, evaluated on the host with the same code the kernels
 * use; lets callers and tests reproduce a draw.  Pure host function. */
float fef_uniform(uint64_t seed, uint32_t position, uint32_t step, uint32_t sequence,
                  uint32_t stream);

/* Measurement aid, not part of the verify path: copy nbytes (a multiple of 16) from src to dst
 * (both device, 16-byte aligned, not overlapping) with a plain streaming kernel of known HBM
 * traffic (nbytes read + nbytes written).  Profiler byte counters are scaled by what they
 * report for this kernel.  Asynchronous on `stream` (hipStream_t, NULL = null stream). */
fef_status fef_copy_probe(void* dst, const void* src, size_t nbytes, void* stream);

/* Measurement aid, not part of the verify path: read nbytes (a multiple of 16) at src (device,
 * 16-byte aligned) once with nothing else to do, in the fastest access pattern found for this
 * machine (128 KB blocks read as 16 rows of 8 KB in bursts of eight 16-byte loads per lane): the
 * rate this gives is the practical ceiling the HBM-bound head kernels are compared with.  `sink` (device,
 * 4 bytes, caller-owned) exists so that the reads have a use; it is written only if the XOR of
 * all words equals one particular value.  Asynchronous on `stream`. */
fef_status fef_read_probe(const void* src, size_t nbytes, void* sink, void* stream);

const char* fef_status_string(fef_status s);
const char* fef_last_error(void);
int32_t fef_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FEF_H */
