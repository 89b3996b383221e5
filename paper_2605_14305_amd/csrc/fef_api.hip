// C ABI of the verify-step library: argument validation, workspace layout, kernel sequencing.
// Everything is validated on the host before the first launch; nothing is allocated.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <atomic>

#include "../../include/fef.h"
#include "fef_device.hpp"

// Scratch of fef_verify_step_static: one copy per GPU the library runs on, held until the process
// ends.  In host code this name is only a handle for hipGetSymbolAddress; the device address it
// yields (one per device) is what kernels, memsets and copies must be given.
static __device__ __align__(256) unsigned char scratch[FEF_STATIC_SCRATCH_BYTES];

namespace {

thread_local char g_err[512] = "";

fef_status fail(fef_status s, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return s;
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct Layout {
  int variant, nT, tile_unit, tile_T, nRC, all_slots;
  long ldl;
  size_t off_logits, off_partials, off_lse, off_xdraft, off_xtarget, off_slot_pos, off_window, off_seqstate,
      off_rmass, off_amass, total;
};

// Sizes only; no pointer checks.
fef_status check_sizes(const fef_params* p, int32_t K, int32_t block) {
  if (!p) return fail(FEF_ERR_INVALID_ARG, "params is NULL");
  if (p->struct_size != sizeof(fef_params))
    return fail(FEF_ERR_INVALID_ARG, "struct_size %u does not match this library's %zu",
                p->struct_size, sizeof(fef_params));
  if (p->B < 1 || p->d < 1 || p->V < 1)
    return fail(FEF_ERR_INVALID_ARG, "B, d, V must be >= 1 (got %d, %d, %d)", p->B, p->d, p->V);
  if (K < 1 || K > FEF_MAX_K || block < 1 || block > FEF_MAX_BLOCK || K > block)
    return fail(FEF_ERR_INVALID_ARG, "need 1 <= K <= min(block, %d) and block <= %d (got K=%d, block=%d)",
                FEF_MAX_K, FEF_MAX_BLOCK, K, block);
  if (p->dtype != FEF_BF16 && p->dtype != FEF_F32)
    return fail(FEF_ERR_INVALID_ARG, "unknown dtype %d", p->dtype);
  if (!(p->temperature > 0.f) || !(p->temperature < 1e30f))
    return fail(FEF_ERR_INVALID_ARG, "temperature must be a positive finite number");
  if (p->dtype == FEF_BF16 && p->d % 64 != 0)
    return fail(FEF_ERR_INVALID_ARG, "bf16 path needs d to be a multiple of 64 (got %d)", p->d);
  if ((long)p->B * K > (1L << 24))
    return fail(FEF_ERR_INVALID_ARG, "B*K = %ld exceeds 2^24 rows per call", (long)p->B * K);
  if (p->lowconf_scope != 0 && p->lowconf_scope != 1)
    return fail(FEF_ERR_INVALID_ARG, "lowconf_scope must be 0 or 1");
  if (p->greedy != 0 && p->greedy != 1) return fail(FEF_ERR_INVALID_ARG, "greedy must be 0 or 1");
  if (!(p->recorrupt_prob > 0.f && p->recorrupt_prob <= 1.f))
    return fail(FEF_ERR_INVALID_ARG, "recorrupt_prob must lie in (0, 1]");
  if (p->phase != FEF_PHASE_FUSED && p->phase != FEF_PHASE_DRAFT && p->phase != FEF_PHASE_TARGET)
    return fail(FEF_ERR_INVALID_ARG, "unknown phase %d", p->phase);
  if (p->seq_pass && p->n_pass < 1)
    return fail(FEF_ERR_INVALID_ARG, "seq_pass needs n_pass >= 1 (got %d)", p->n_pass);
  if (!p->conf && (p->pass_mask || p->lowconf_scope == 1))
    return fail(FEF_ERR_INVALID_ARG, "conf may be NULL only with pass_mask NULL and lowconf_scope 0");
  return FEF_OK;
}

fef_status select_variant(const fef_params* p, int32_t K, int* variant) {
  const long M = (p->phase == FEF_PHASE_FUSED ? 2L : 1L) * p->B * K;  // rows through the head in this call
  int v = p->gemm_variant;
  if (v == FEF_GEMM_AUTO) {
    if (p->dtype == FEF_F32) v = FEF_GEMM_F32;
    else if (fef::skinny_supports((int)(M > 1 << 20 ? 1 << 20 : M), p->d)) v = FEF_GEMM_SKINNY;
    else if (M > 128) v = FEF_GEMM_TILED256;
    else if (!fef::rowstream_supports((int)M, p->d)) v = FEF_GEMM_STREAM;
    else if (M <= 48 || (M > 64 && M <= 96)) {
      // the row-streaming kernel works on 64, 96 or 128 rows, the LDS-streaming one on 64 or 128: where the
      // first needs fewer it is ahead (whole step at d = 4096, V = 126464: 219 against 222 us at M = 48, 253
      // against 266 at M = 96), where both need the same the second is (219.5 against 224 us at M = 64)
      v = FEF_GEMM_ROWSTREAM;
    } else {
      // 48 < M <= 64 and 96 < M <= 128 (216 against 242 us at M = 128; also at V = 151936, which divides
      // better into the other kernel's rounds of tiles: 272 against 275 us)
      v = FEF_GEMM_STREAM;
    }
  }
  switch (v) {
    case FEF_GEMM_SKINNY:
      if (p->dtype != FEF_BF16 || !fef::skinny_supports((int)(M > 1 << 20 ? 1 << 20 : M), p->d))
        return fail(FEF_ERR_UNSUPPORTED, "skinny head kernel needs bf16, at most 32 rows through the head and d in {512, 1024, 2048, 2560, 3072, 3584, 4096}");
      break;
    case FEF_GEMM_TILED:
    case FEF_GEMM_TILED256:
      if (p->dtype != FEF_BF16) return fail(FEF_ERR_UNSUPPORTED, "tiled head kernels are bf16 only");
      break;
    case FEF_GEMM_STREAM:
      if (p->dtype != FEF_BF16 || !fef::stream_supports((int)(M > 1 << 20 ? 1 << 20 : M), p->d))
        return fail(FEF_ERR_UNSUPPORTED, "streaming head kernel needs bf16 and at most 128 rows through the head");
      break;
    case FEF_GEMM_ROWSTREAM:
      if (p->dtype != FEF_BF16 || !fef::rowstream_supports((int)(M > 1 << 20 ? 1 << 20 : M), p->d))
        return fail(FEF_ERR_UNSUPPORTED, "row-streaming head kernel needs bf16, at most 128 rows through the head and d a multiple of 512");
      break;
    case FEF_GEMM_F32:
      if (p->dtype != FEF_F32) return fail(FEF_ERR_UNSUPPORTED, "f32 head kernel needs dtype f32");
      if (M > 65535) return fail(FEF_ERR_UNSUPPORTED, "f32 head kernel serves at most 65535 rows");
      break;
    default:
      return fail(FEF_ERR_INVALID_ARG, "unknown gemm_variant %d", v);
  }
  *variant = v;
  return FEF_OK;
}

fef_status make_layout(const fef_params* p, int32_t K, int32_t block, Layout* L) {
  fef_status s = check_sizes(p, K, block);
  if (s != FEF_OK) return s;
  s = select_variant(p, K, &L->variant);
  if (s != FEF_OK) return s;
  const size_t BK = (size_t)p->B * K, M = 2 * BK;
  if (L->variant == FEF_GEMM_SKINNY) {
    // one partial per (row, workgroup); a workgroup's tokens are a contiguous run of 16-token tiles
    L->tile_unit = fef::kSkinnyUnit;
    L->tile_T = (p->V + fef::kSkinnyUnit - 1) / fef::kSkinnyUnit;
    L->nT = L->tile_T < fef::kSkinnyMaxGrid ? L->tile_T : fef::kSkinnyMaxGrid;
  } else if (L->variant == FEF_GEMM_ROWSTREAM) {
    // as above, with this kernel's grid
    L->tile_unit = fef::kSkinnyUnit;
    L->tile_T = (p->V + fef::kSkinnyUnit - 1) / fef::kSkinnyUnit;
    L->nT = fef::rowstream_grid(p->V);
  } else if (L->variant == FEF_GEMM_STREAM) {
    // one partial per (row, workgroup); a workgroup's tokens are a contiguous run of 64-token units
    L->tile_unit = fef::kTiledTn;
    L->tile_T = (p->V + fef::kTiledTn - 1) / fef::kTiledTn;
    L->nT = fef::stream_grid(p->V);
  } else if (L->variant == FEF_GEMM_TILED256) {
    // one partial per (row, workgroup tile of 256 tokens)
    L->tile_unit = fef::kTiled256Tn;
    L->tile_T = L->nT = (p->V + fef::kTiled256Tn - 1) / fef::kTiled256Tn;
  } else {
    L->tile_unit = fef::kTiledTn;
    L->tile_T = L->nT = (p->V + fef::kTiledTn - 1) / fef::kTiledTn;
  }
  L->nRC = (p->V + fef::kResidChunk - 1) / fef::kResidChunk;
  L->ldl = (long)align_up((size_t)p->V, 64);
  L->all_slots = (p->diag_alpha || p->diag_resid_mass) ? 1 : 0;
  const size_t nslots = L->all_slots ? BK : (size_t)p->B;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
  L->off_logits = take(M * (size_t)L->ldl * sizeof(float));
  L->off_partials = take(M * (size_t)L->nT * sizeof(float2));
  L->off_lse = take(M * sizeof(float));
  L->off_xdraft = take(BK * sizeof(int32_t));
  L->off_xtarget = take(BK * sizeof(int32_t));
  L->off_slot_pos = take(BK * sizeof(int32_t));
  L->off_window = take((size_t)p->B * sizeof(int32_t));
  L->off_seqstate = take((size_t)p->B * sizeof(fef::SeqState));
  L->off_rmass = take(nslots * (size_t)L->nRC * sizeof(float));
  L->off_amass = take(L->all_slots ? nslots * (size_t)L->nRC * sizeof(float) : 0);
  L->total = o;
  return FEF_OK;
}

__global__ __launch_bounds__(256) void copy_probe_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src,
                                                        size_t n16) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = src[i];
}

// The fastest read of a large buffer found on this machine, which is what the probe is for: the
// buffer as blocks of 16 rows of 8 KB (the shape of a 16-token tile of W at d = 4096); one workgroup
// per CU walks a contiguous run of blocks; its eight wavefronts split a row eight ways, and a
// wavefront fetches its 1 KB of each of the 16 rows in two bursts of eight 16-byte loads per lane
// (16 rows x 64 bytes per load), the last 64 bytes of a burst first, the next burst requested before
// the one in hand is consumed and waited for in full before anything else is asked for.  6.6 TB/s
// on 1 GB; a linear sweep with eight loads per thread in flight reaches 6.1 to 6.2.  What does not
// fill a block is swept linearly.
__global__ __launch_bounds__(512) void read_probe_kernel(const char* __restrict__ src, size_t nbytes, unsigned* sink) {
  constexpr size_t kBlock = 16 * 8192;
  const size_t nblocks = nbytes / kBlock;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int i16 = lane & 15, g = lane >> 4;
  const size_t b0 = blockIdx.x * nblocks / gridDim.x, b1 = (blockIdx.x + 1) * nblocks / gridDim.x;
  const size_t nburst = 2 * (b1 - b0);
  uint4 acc = {0u, 0u, 0u, 0u};
  auto burst = [&](size_t j, uint4(&v)[8]) {
    const char* p = src + (b0 + (j >> 1)) * kBlock + (size_t)i16 * 8192 + wave * 1024 + g * 16 + (j & 1) * 512;
    v[7] = *reinterpret_cast<const uint4*>(p + 448);
    asm volatile("" ::: "memory");
#pragma unroll
    for (int u = 0; u < 7; ++u) {
      v[u] = *reinterpret_cast<const uint4*>(p + 64 * u);
      asm volatile("" ::: "memory");
    }
  };
  uint4 cur[8], nxt[8];
  if (nburst) burst(0, cur);
  for (size_t j = 0; j < nburst; ++j) {
    burst(j + 1 < nburst ? j + 1 : j, nxt);
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      acc.x ^= cur[u].x; acc.y ^= cur[u].y; acc.z ^= cur[u].z; acc.w ^= cur[u].w;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) cur[u] = nxt[u];
  }
  const uint4* tail = reinterpret_cast<const uint4*>(src + nblocks * kBlock);
  const size_t ntail = (nbytes - nblocks * kBlock) / 16;
  for (size_t i = (size_t)blockIdx.x * 512 + threadIdx.x; i < ntail; i += (size_t)gridDim.x * 512) {
    const uint4 v = tail[i];
    acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w;
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9E3779B9u) *sink = 1u;
}

}  // namespace

extern "C" {

fef_status fef_read_probe(const void* src, size_t nbytes, void* sink, void* stream) {
  if (!src || !sink || nbytes == 0 || nbytes % 16 || ((uintptr_t)src & 15) || ((uintptr_t)sink & 3))
    return fail(FEF_ERR_INVALID_ARG, "read probe needs a non-NULL 16-byte aligned source, a size multiple of 16 and a sink");
  hipLaunchKernelGGL(read_probe_kernel, dim3(256), dim3(512), 0, (hipStream_t)stream, (const char*)src, nbytes,
                     (unsigned*)sink);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(FEF_ERR_HIP, "read probe launch: %s", hipGetErrorString(e));
  return FEF_OK;
}

fef_status fef_copy_probe(void* dst, const void* src, size_t nbytes, void* stream) {
  if (!dst || !src || nbytes == 0 || nbytes % 16 || (((uintptr_t)dst | (uintptr_t)src) & 15))
    return fail(FEF_ERR_INVALID_ARG, "copy probe needs non-NULL 16-byte aligned pointers and a size multiple of 16");
  hipLaunchKernelGGL(copy_probe_kernel, dim3(2048), dim3(256), 0, (hipStream_t)stream, (uint4*)dst,
                     (const uint4*)src, nbytes / 16);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(FEF_ERR_HIP, "copy probe launch: %s", hipGetErrorString(e));
  return FEF_OK;
}

size_t fef_workspace_bytes(const fef_params* prm, int32_t K, int32_t block) {
  Layout L;
  if (make_layout(prm, K, block, &L) != FEF_OK) return 0;
  return L.total;
}

int32_t fef_select_gemm(const fef_params* prm, int32_t K) {
  fef_status s = check_sizes(prm, K, K > 0 ? (K > FEF_MAX_BLOCK ? FEF_MAX_BLOCK : K) : 1);
  if (s != FEF_OK) return s;
  int v = 0;
  s = select_variant(prm, K, &v);
  return s != FEF_OK ? (int32_t)s : v;
}

namespace {
constexpr int kPhaseTopN = 3;  // internal: draft rows only, then the baseline's top-n selection
fef_status run_step(const fef_params* prm, int phase, int n_transfer, const void* h_draft, const void* h_target,
                    const void* W_vocab, int32_t K, int32_t block, uint64_t seed, int32_t* out_tokens,
                    int32_t* out_accept_len, uint8_t* out_remask, void* workspace, size_t workspace_bytes);
}  // namespace

fef_status fef_verify_step(const fef_params* prm, const void* h_draft, const void* h_target,
                           const void* W_vocab, int32_t K, int32_t block, uint64_t seed,
                           int32_t* out_tokens, int32_t* out_accept_len, uint8_t* out_remask) {
  if (!prm) return fail(FEF_ERR_INVALID_ARG, "params is NULL");
  return run_step(prm, prm->phase, 0, h_draft, h_target, W_vocab, K, block, seed, out_tokens, out_accept_len,
                  out_remask, prm->workspace, prm->workspace_bytes);
}

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];  // device address of `scratch` per device, NULL = not asked yet

// Address of this device's copy of `scratch`; resolved once per device with that device current.
fef_status static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(FEF_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return fail(FEF_ERR_UNSUPPORTED, "device index %d out of range", dev);
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!ptr) {
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr)
      return fail(FEF_ERR_HIP, "hipGetSymbolAddress(scratch) on device %d: %s", dev, hipGetErrorString(e));
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);  // concurrent first calls store the same address
  }
  *out = ptr;
  return FEF_OK;
}
}  // namespace

fef_status fef_verify_step_static(const fef_params* prm, const void* h_draft, const void* h_target,
                                  const void* W_vocab, int32_t K, int32_t block, uint64_t seed,
                                  int32_t* out_tokens, int32_t* out_accept_len, uint8_t* out_remask) {
  if (!prm) return fail(FEF_ERR_INVALID_ARG, "params is NULL");
  Layout L;
  fef_status s = make_layout(prm, K, block, &L);
  if (s != FEF_OK) return s;
  if (L.total > (size_t)FEF_STATIC_SCRATCH_BYTES)
    return fail(FEF_ERR_WORKSPACE, "this call needs %zu bytes of scratch, the built-in buffer has %zu: use fef_verify_step "
                "with a caller workspace", L.total, (size_t)FEF_STATIC_SCRATCH_BYTES);
  void* ptr = nullptr;
  s = static_scratch(&ptr);
  if (s != FEF_OK) return s;
  return run_step(prm, prm->phase, 0, h_draft, h_target, W_vocab, K, block, seed, out_tokens, out_accept_len,
                  out_remask, ptr, (size_t)FEF_STATIC_SCRATCH_BYTES);
}

fef_status fef_topn_step(const fef_params* prm, const void* h, const void* W_vocab, int32_t K, int32_t block,
                         uint64_t seed, int32_t n_transfer, int32_t* out_tokens, int32_t* out_committed,
                         uint8_t* out_remask) {
  if (!prm) return fail(FEF_ERR_INVALID_ARG, "params is NULL");
  if (n_transfer < 1) return fail(FEF_ERR_INVALID_ARG, "n_transfer must be at least 1 (got %d)", n_transfer);
  if (prm->phase != FEF_PHASE_FUSED) return fail(FEF_ERR_INVALID_ARG, "phase must be FUSED (0) in a baseline step");
  if (prm->draft_tokens || prm->pass_mask || prm->seq_pass || prm->seq_rounds)
    return fail(FEF_ERR_INVALID_ARG, "draft_tokens, pass_mask, seq_pass and seq_rounds have no meaning in a baseline step");
  fef_params p = *prm;
  p.phase = FEF_PHASE_DRAFT;  // sizes, kernel choice and workspace layout of a call over B*K rows
  return run_step(&p, kPhaseTopN, n_transfer, h, nullptr, W_vocab, K, block, seed, out_tokens, out_committed,
                  out_remask, p.workspace, p.workspace_bytes);
}

namespace {
fef_status run_step(const fef_params* prm, int phase, int n_transfer, const void* h_draft, const void* h_target,
                    const void* W_vocab, int32_t K, int32_t block, uint64_t seed, int32_t* out_tokens,
                    int32_t* out_accept_len, uint8_t* out_remask, void* workspace, size_t workspace_bytes) {
  Layout L;
  fef_status s = make_layout(prm, K, block, &L);
  if (s != FEF_OK) return s;
  if ((!h_draft && phase != FEF_PHASE_TARGET) || (!h_target && phase != FEF_PHASE_DRAFT && phase != kPhaseTopN) ||
      !W_vocab)
    return fail(FEF_ERR_INVALID_ARG, "h_draft, h_target and W_vocab must not be NULL");
  if (!out_tokens || ((!out_accept_len || !out_remask) && phase != FEF_PHASE_DRAFT))
    return fail(FEF_ERR_INVALID_ARG, "out_tokens, out_accept_len and out_remask must not be NULL");
  if (((uintptr_t)h_draft | (uintptr_t)h_target | (uintptr_t)W_vocab) & 15)
    return fail(FEF_ERR_INVALID_ARG, "h_draft, h_target and W_vocab must be 16-byte aligned");
  if (!prm->ev_head_begin != !prm->ev_head_end)
    return fail(FEF_ERR_INVALID_ARG, "ev_head_begin and ev_head_end must be given together");
  if (!workspace) return fail(FEF_ERR_WORKSPACE, "workspace is NULL (%zu bytes needed)", L.total);
  if ((uintptr_t)workspace & 255) return fail(FEF_ERR_WORKSPACE, "workspace must be 256-byte aligned");
  if (workspace_bytes < L.total)
    return fail(FEF_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, L.total);

  char* ws = (char*)workspace;
  hipStream_t stream = (hipStream_t)prm->stream;

  fef::HeadArgs h{};
  h.h_draft = h_draft; h.h_target = h_target; h.W = W_vocab;
  h.BK = prm->B * K; h.d = prm->d; h.V = prm->V;
  h.row0 = phase == FEF_PHASE_TARGET ? h.BK : 0;
  h.nrows = phase == FEF_PHASE_FUSED ? 2 * h.BK : h.BK;
  h.inv_tau = 1.0f / prm->temperature;
  h.logits = (float*)(ws + L.off_logits) + (size_t)h.row0 * L.ldl; h.ldl = L.ldl;
  h.partials = (float2*)(ws + L.off_partials) + (size_t)h.row0 * L.nT; h.nT = L.nT;
  h.stream = stream;
  h.ev_begin = (hipEvent_t)prm->ev_head_begin; h.ev_end = (hipEvent_t)prm->ev_head_end;
  hipError_t e;
  switch (L.variant) {
    case FEF_GEMM_SKINNY: e = fef::launch_head_skinny(h); break;
    case FEF_GEMM_TILED: e = fef::launch_head_tiled(h); break;
    case FEF_GEMM_TILED256: e = fef::launch_head_tiled256(h); break;
    case FEF_GEMM_STREAM: e = fef::launch_head_stream(h); break;
    case FEF_GEMM_ROWSTREAM: e = fef::launch_head_rowstream(h); break;
    default: e = fef::launch_head_f32(h); break;
  }
  if (e != hipSuccess) return fail(FEF_ERR_HIP, "head kernel launch: %s", hipGetErrorString(e));

  fef::VerifyArgs v;
  memset(&v, 0, sizeof v);
  v.B = prm->B; v.K = K; v.block = block; v.V = prm->V;
  v.row0 = h.row0; v.nrows = h.nrows; v.phase = phase;
  v.ldl = L.ldl; v.logits = (float*)(ws + L.off_logits); v.partials = (float2*)(ws + L.off_partials); v.nT = L.nT;
  v.tile_unit = L.tile_unit; v.tile_T = L.tile_T; v.tile_G = L.nT;
  v.seed = seed; v.step = prm->step; v.seq_base = prm->seq_base; v.pos_base = prm->pos_base;
  v.n_rm = prm->n_rm; v.final_pass = prm->final_pass; v.lowconf_scope = prm->lowconf_scope;
  v.recorrupt_prob = prm->recorrupt_prob;
  v.greedy = prm->greedy;
  v.mask_in = prm->mask_in; v.pass_mask = prm->pass_mask; v.conf = prm->conf;
  v.draft_tokens_in = prm->draft_tokens;
  v.n_pass = prm->n_pass; v.seq_pass = prm->seq_pass; v.seq_rounds = prm->seq_rounds;
  v.tokens_state = prm->tokens_state;
  v.lse = (float*)(ws + L.off_lse);
  v.xdraft = (int32_t*)(ws + L.off_xdraft);
  v.xtarget = (int32_t*)(ws + L.off_xtarget);
  v.slot_pos = (int32_t*)(ws + L.off_slot_pos);
  v.window = (int32_t*)(ws + L.off_window);
  v.seqstate = (fef::SeqState*)(ws + L.off_seqstate);
  v.rmass = (float*)(ws + L.off_rmass);
  v.amass = (float*)(ws + L.off_amass);
  v.nRC = L.nRC; v.all_slots = L.all_slots;
  v.out_tokens = out_tokens; v.out_accept_len = out_accept_len; v.out_remask = out_remask;
  v.diag_draft_tokens = prm->diag_draft_tokens; v.diag_alpha = prm->diag_alpha;
  v.diag_resid_mass = prm->diag_resid_mass; v.diag_lse = prm->diag_lse;
  v.diag_logits = prm->diag_logits; v.diag_conf_tok = prm->diag_conf_tok;
  v.stream = stream;
  v.n_transfer = n_transfer;
  e = fef::launch_verify(v);
  if (e != hipSuccess) return fail(FEF_ERR_HIP, "verify kernel launch: %s", hipGetErrorString(e));
  return FEF_OK;
}
}  // namespace

namespace {
// sizes and kernel choice of a cross-entropy call; *variant receives the head kernel
fef_status ce_check(const fef_params* p, int32_t R, int* variant, int* nT, size_t* total) {
  if (!p) return fail(FEF_ERR_INVALID_ARG, "params is NULL");
  if (p->struct_size != sizeof(fef_params))
    return fail(FEF_ERR_INVALID_ARG, "struct_size %u does not match this library's %zu", p->struct_size,
                sizeof(fef_params));
  if (R < 1 || R > (1 << 24)) return fail(FEF_ERR_INVALID_ARG, "R = %d out of range [1, 2^24]", R);
  if (p->V < 1 || p->d < 1) return fail(FEF_ERR_INVALID_ARG, "V and d must be positive");
  if (p->dtype != FEF_BF16 && p->dtype != FEF_F32) return fail(FEF_ERR_INVALID_ARG, "unknown dtype %d", p->dtype);
  if (p->dtype == FEF_BF16 && p->d % 64 != 0)
    return fail(FEF_ERR_INVALID_ARG, "bf16 needs d to be a multiple of 64 (got %d)", p->d);
  if (!(p->temperature > 0.f) || !(p->temperature < INFINITY))
    return fail(FEF_ERR_INVALID_ARG, "temperature must be positive and finite");
  int v = p->gemm_variant;
  if (v == FEF_GEMM_AUTO)
    v = p->dtype == FEF_F32 ? FEF_GEMM_F32 : R <= 128 ? FEF_GEMM_STREAM : FEF_GEMM_TILED256;
  switch (v) {
    case FEF_GEMM_F32:
      if (p->dtype != FEF_F32) return fail(FEF_ERR_UNSUPPORTED, "f32 head kernel needs dtype f32");
      if (R > 65535) return fail(FEF_ERR_UNSUPPORTED, "f32 head kernel serves at most 65535 rows");
      break;
    case FEF_GEMM_STREAM:
      if (p->dtype != FEF_BF16 || !fef::stream_supports(R, p->d))
        return fail(FEF_ERR_UNSUPPORTED, "streaming head kernel needs bf16 and at most 128 rows");
      break;
    case FEF_GEMM_TILED256:
      if (p->dtype != FEF_BF16) return fail(FEF_ERR_UNSUPPORTED, "tiled head kernels are bf16 only");
      break;
    default:
      return fail(FEF_ERR_UNSUPPORTED, "cross-entropy runs through the F32, STREAM or TILED256 head kernel");
  }
  *variant = v;
  *nT = v == FEF_GEMM_STREAM     ? fef::stream_grid(p->V)
        : v == FEF_GEMM_TILED256 ? (p->V + fef::kTiled256Tn - 1) / fef::kTiled256Tn
                                 : (p->V + fef::kTiledTn - 1) / fef::kTiledTn;
  *total = align_up((size_t)R * (size_t)*nT * sizeof(float2), 256) + align_up((size_t)R * sizeof(float), 256);
  return FEF_OK;
}
}  // namespace

size_t fef_cross_entropy_workspace_bytes(const fef_params* prm, int32_t R) {
  int v, nT;
  size_t total;
  return ce_check(prm, R, &v, &nT, &total) == FEF_OK ? total : 0;
}

fef_status fef_head_cross_entropy(const fef_params* prm, const void* h, const void* W_vocab,
                                  const int32_t* labels, int32_t R, float* out_ce, float* out_loss) {
  int variant, nT;
  size_t total;
  fef_status s = ce_check(prm, R, &variant, &nT, &total);
  if (s != FEF_OK) return s;
  if (!h || !W_vocab || !labels || !out_ce)
    return fail(FEF_ERR_INVALID_ARG, "h, W_vocab, labels and out_ce must not be NULL");
  if (((uintptr_t)h | (uintptr_t)W_vocab) & 15)
    return fail(FEF_ERR_INVALID_ARG, "h and W_vocab must be 16-byte aligned");
  if (!prm->ev_head_begin != !prm->ev_head_end)
    return fail(FEF_ERR_INVALID_ARG, "ev_head_begin and ev_head_end must be given together");
  if (!prm->workspace) return fail(FEF_ERR_WORKSPACE, "workspace is NULL (%zu bytes needed)", total);
  if ((uintptr_t)prm->workspace & 255) return fail(FEF_ERR_WORKSPACE, "workspace must be 256-byte aligned");
  if (prm->workspace_bytes < total)
    return fail(FEF_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", prm->workspace_bytes, total);

  char* ws = (char*)prm->workspace;
  fef::HeadArgs a{};
  a.h_draft = h; a.h_target = h; a.W = W_vocab;
  a.BK = R; a.d = prm->d; a.V = prm->V; a.row0 = 0; a.nrows = R;
  a.inv_tau = 1.0f / prm->temperature;
  a.logits = nullptr; a.ldl = 0;
  a.partials = (float2*)ws; a.nT = nT;
  a.labels = labels;
  a.label_logit = (float*)(ws + align_up((size_t)R * (size_t)nT * sizeof(float2), 256));
  a.stream = (hipStream_t)prm->stream;
  a.ev_begin = (hipEvent_t)prm->ev_head_begin; a.ev_end = (hipEvent_t)prm->ev_head_end;
  hipError_t e = fef::launch_ce_init(a.label_logit, R, a.stream);
  if (e != hipSuccess) return fail(FEF_ERR_HIP, "cross-entropy kernel launch: %s", hipGetErrorString(e));
  switch (variant) {
    case FEF_GEMM_TILED256: e = fef::launch_head_tiled256(a); break;
    case FEF_GEMM_STREAM: e = fef::launch_head_stream(a); break;
    default: e = fef::launch_head_f32(a); break;
  }
  if (e != hipSuccess) return fail(FEF_ERR_HIP, "head kernel launch: %s", hipGetErrorString(e));
  fef::CeArgs c{};
  c.R = R; c.nT = nT; c.partials = a.partials; c.labels = labels; c.label_logit = a.label_logit;
  c.out_ce = out_ce; c.out_loss = out_loss; c.stream = a.stream;
  e = fef::launch_ce_finish(c);
  if (e != hipSuccess) return fail(FEF_ERR_HIP, "cross-entropy kernel launch: %s", hipGetErrorString(e));
  return FEF_OK;
}

float fef_uniform(uint64_t seed, uint32_t position, uint32_t step, uint32_t sequence, uint32_t stream) {
  return fef::philox_uniform(seed, position, step, sequence, stream);
}

const char* fef_status_string(fef_status s) {
  switch (s) {
    case FEF_OK: return "ok";
    case FEF_ERR_INVALID_ARG: return "invalid argument";
    case FEF_ERR_UNSUPPORTED: return "unsupported configuration";
    case FEF_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case FEF_ERR_HIP: return "HIP runtime error";
  }
  return "unknown status";
}

const char* fef_last_error(void) { return g_err; }

int32_t fef_abi_version(void) { return FEF_ABI_VERSION; }

}  // extern "C"
