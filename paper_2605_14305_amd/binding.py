"""ctypes binding of libfef.so (see include/fef.h).  Argument marshalling only: every step of
the verify path runs in the library's HIP kernels.  PyTorch supplies device memory and the
current stream.  There is no fallback: if the library has not been built, loading raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("FEF_LIB") or os.path.join(_HERE, "libfef.so")  # FEF_LIB: another build of the same library

FEF_OK = 0
FEF_ERR_INVALID_ARG = -1
FEF_ERR_UNSUPPORTED = -2
FEF_ERR_WORKSPACE = -3
FEF_ERR_HIP = -4
FEF_BF16, FEF_F32 = 0, 1
FEF_GEMM_AUTO, FEF_GEMM_SKINNY, FEF_GEMM_TILED, FEF_GEMM_F32, FEF_GEMM_TILED256, FEF_GEMM_STREAM = 0, 1, 2, 3, 4, 5
FEF_GEMM_ROWSTREAM = 6
FEF_MAX_K, FEF_MAX_BLOCK = 64, 4096
FEF_PHASE_FUSED, FEF_PHASE_DRAFT, FEF_PHASE_TARGET = 0, 1, 2

ABI_VERSION = 10   # FEF_ABI_VERSION of include/fef.h this binding's fef_params mirrors

EXPORTS = ["fef_workspace_bytes", "fef_verify_step", "fef_select_gemm", "fef_uniform",
           "fef_status_string", "fef_last_error", "fef_abi_version", "fef_copy_probe", "fef_read_probe",
           "fef_cross_entropy_workspace_bytes", "fef_head_cross_entropy", "fef_topn_step",
           "fef_verify_step_static"]
FEF_STATIC_SCRATCH_BYTES = 32 << 20


class fef_params(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32),
        ("B", ctypes.c_int32), ("d", ctypes.c_int32), ("V", ctypes.c_int32),
        ("dtype", ctypes.c_int32),
        ("temperature", ctypes.c_float),
        ("step", ctypes.c_uint32), ("seq_base", ctypes.c_uint32), ("pos_base", ctypes.c_uint32),
        ("n_rm", ctypes.c_int32), ("final_pass", ctypes.c_int32),
        ("lowconf_scope", ctypes.c_int32), ("gemm_variant", ctypes.c_int32),
        ("mask_in", ctypes.c_void_p), ("pass_mask", ctypes.c_void_p), ("conf", ctypes.c_void_p),
        ("draft_tokens", ctypes.c_void_p),
        ("diag_draft_tokens", ctypes.c_void_p), ("diag_alpha", ctypes.c_void_p),
        ("diag_resid_mass", ctypes.c_void_p), ("diag_lse", ctypes.c_void_p),
        ("diag_logits", ctypes.c_void_p), ("diag_conf_tok", ctypes.c_void_p),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
        ("stream", ctypes.c_void_p),
        ("ev_head_begin", ctypes.c_void_p), ("ev_head_end", ctypes.c_void_p),
        ("n_pass", ctypes.c_int32), ("seq_pass", ctypes.c_void_p), ("seq_rounds", ctypes.c_void_p),
        ("tokens_state", ctypes.c_void_p), ("phase", ctypes.c_int32),
        ("recorrupt_prob", ctypes.c_float), ("greedy", ctypes.c_int32),
    ]


class FefError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"fef status {status}: {message}")
        self.status = status


_lib = None


def lib():
    """Load libfef.so once.  Raises if it has not been built (python -m paper_2605_14305_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} not found: build it with `python -m paper_2605_14305_amd.build`; "
                "there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        L.fef_workspace_bytes.restype = ctypes.c_size_t
        L.fef_workspace_bytes.argtypes = [ctypes.POINTER(fef_params), ctypes.c_int32, ctypes.c_int32]
        L.fef_verify_step.restype = ctypes.c_int
        L.fef_verify_step.argtypes = [ctypes.POINTER(fef_params), ctypes.c_void_p, ctypes.c_void_p,
                                      ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_uint64,
                                      ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        L.fef_verify_step_static.restype = ctypes.c_int
        L.fef_verify_step_static.argtypes = L.fef_verify_step.argtypes
        L.fef_select_gemm.restype = ctypes.c_int32
        L.fef_select_gemm.argtypes = [ctypes.POINTER(fef_params), ctypes.c_int32]
        L.fef_uniform.restype = ctypes.c_float
        L.fef_uniform.argtypes = [ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint32,
                                  ctypes.c_uint32]
        L.fef_status_string.restype = ctypes.c_char_p
        L.fef_status_string.argtypes = [ctypes.c_int]
        L.fef_last_error.restype = ctypes.c_char_p
        L.fef_last_error.argtypes = []
        L.fef_copy_probe.restype = ctypes.c_int
        L.fef_copy_probe.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        L.fef_read_probe.restype = ctypes.c_int
        L.fef_read_probe.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
        L.fef_abi_version.restype = ctypes.c_int32
        L.fef_abi_version.argtypes = []
        L.fef_cross_entropy_workspace_bytes.restype = ctypes.c_size_t
        L.fef_cross_entropy_workspace_bytes.argtypes = [ctypes.POINTER(fef_params), ctypes.c_int32]
        L.fef_topn_step.restype = ctypes.c_int
        L.fef_topn_step.argtypes = [ctypes.POINTER(fef_params), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32,
                                    ctypes.c_int32, ctypes.c_uint64, ctypes.c_int32, ctypes.c_void_p,
                                    ctypes.c_void_p, ctypes.c_void_p]
        L.fef_head_cross_entropy.restype = ctypes.c_int
        L.fef_head_cross_entropy.argtypes = [ctypes.POINTER(fef_params), ctypes.c_void_p, ctypes.c_void_p,
                                             ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p]
        if L.fef_abi_version() != ABI_VERSION:
            raise RuntimeError(f"{LIB_PATH} has ABI version {L.fef_abi_version()}, this binding needs {ABI_VERSION}: "
                               "rebuild it with `python -m paper_2605_14305_amd.build`")
        _lib = L
    return _lib


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def make_params(B, d, V, dtype=FEF_BF16, temperature=1.0, step=0, seq_base=0, pos_base=0,
                n_rm=-1, final_pass=0, lowconf_scope=0, gemm_variant=FEF_GEMM_AUTO):
    p = fef_params()
    p.struct_size = ctypes.sizeof(fef_params)
    p.B, p.d, p.V, p.dtype = B, d, V, dtype
    p.temperature = temperature
    p.step, p.seq_base, p.pos_base = step, seq_base, pos_base
    p.n_rm, p.final_pass, p.lowconf_scope, p.gemm_variant = n_rm, int(final_pass), lowconf_scope, gemm_variant
    p.recorrupt_prob = 1.0
    return p


def fef_workspace_bytes(params, K, block):
    return lib().fef_workspace_bytes(ctypes.byref(params), K, block)


def fef_select_gemm(params, K):
    return lib().fef_select_gemm(ctypes.byref(params), K)


def fef_uniform(seed, position, step, sequence, stream):
    return lib().fef_uniform(seed, position, step, sequence, stream)


def fef_last_error():
    return lib().fef_last_error().decode()


def fef_verify_step(params, h_draft, h_target, W_vocab, K, block, seed, out_tokens, out_accept_len,
                    out_remask):
    """Raw call: tensors (or None) are passed as device pointers; raises FefError on failure."""
    s = lib().fef_verify_step(ctypes.byref(params), _ptr(h_draft), _ptr(h_target), _ptr(W_vocab), K,
                              block, ctypes.c_uint64(seed & 0xFFFFFFFFFFFFFFFF), _ptr(out_tokens),
                              _ptr(out_accept_len), _ptr(out_remask))
    if s != FEF_OK:
        raise FefError(s, fef_last_error())
    return s


def fef_verify_step_static(params, h_draft, h_target, W_vocab, K, block, seed, out_tokens, out_accept_len,
                           out_remask):
    """fef_verify_step on the library's built-in scratch buffer: no workspace, no allocation."""
    s = lib().fef_verify_step_static(ctypes.byref(params), _ptr(h_draft), _ptr(h_target), _ptr(W_vocab), K,
                                     block, ctypes.c_uint64(seed & 0xFFFFFFFFFFFFFFFF), _ptr(out_tokens),
                                     _ptr(out_accept_len), _ptr(out_remask))
    if s != FEF_OK:
        raise FefError(s, fef_last_error())
    return s


def fef_copy_probe(dst, src):
    """Plain device copy of known traffic (profiler counter calibration)."""
    assert dst.numel() * dst.element_size() == src.numel() * src.element_size()
    s = lib().fef_copy_probe(_ptr(dst), _ptr(src), src.numel() * src.element_size(),
                             ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    if s != FEF_OK:
        raise FefError(s, fef_last_error())


def fef_read_probe(src, sink):
    """Plain streaming read of `src` (the practical HBM read ceiling); `sink` is a 4-byte device tensor."""
    s = lib().fef_read_probe(_ptr(src), src.numel() * src.element_size(), _ptr(sink),
                             ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    if s != FEF_OK:
        raise FefError(s, fef_last_error())


class HeadCrossEntropy:
    """Token-level cross-entropy of R rows through the vocabulary head (fef_head_cross_entropy);
    holds workspace and outputs of one shape so that repeated calls do no allocation."""

    def __init__(self, R, d, V, dtype="bf16", device="cuda", gemm_variant=FEF_GEMM_AUTO):
        self.R, self.d, self.V, self.device = R, d, V, torch.device(device)
        self.dtype = FEF_BF16 if dtype == "bf16" else FEF_F32
        self.torch_dtype = torch.bfloat16 if dtype == "bf16" else torch.float32
        self.gemm_variant = gemm_variant
        n = lib().fef_cross_entropy_workspace_bytes(ctypes.byref(self._params()), R)
        if n == 0:
            raise FefError(FEF_ERR_INVALID_ARG, fef_last_error())
        self.workspace = torch.empty(n, dtype=torch.uint8, device=self.device)
        self.out_ce = torch.empty(R, dtype=torch.float32, device=self.device)
        self.out_loss = torch.empty(1, dtype=torch.float32, device=self.device)

    def _params(self, temperature=1.0):
        return make_params(1, self.d, self.V, dtype=self.dtype, temperature=temperature,
                           gemm_variant=self.gemm_variant)

    def __call__(self, h, W_vocab, labels, temperature=1.0, head_events=None):
        assert tuple(h.shape) == (self.R, self.d) and tuple(W_vocab.shape) == (self.V, self.d)
        assert h.dtype == self.torch_dtype and W_vocab.dtype == self.torch_dtype
        assert labels.dtype == torch.int32 and tuple(labels.shape) == (self.R,)
        for t in (h, W_vocab, labels):
            assert t.is_contiguous() and t.device.type == "cuda"
        p = self._params(temperature)
        p.workspace = self.workspace.data_ptr()
        p.workspace_bytes = self.workspace.numel()
        p.stream = torch.cuda.current_stream(self.device).cuda_stream
        if head_events is not None:
            p.ev_head_begin, p.ev_head_end = head_events
        s = lib().fef_head_cross_entropy(ctypes.byref(p), _ptr(h), _ptr(W_vocab), _ptr(labels), self.R,
                                         _ptr(self.out_ce), _ptr(self.out_loss))
        if s != FEF_OK:
            raise FefError(s, fef_last_error())
        return self.out_ce, self.out_loss


class VerifyStep:
    """Holds the output and workspace tensors of one problem shape so that repeated calls do no
    allocation.  `diag=True` also returns draft tokens, alpha, residual mass, lse, confidences
    (and logits with diag_logits=True)."""

    def __init__(self, B, K, block, d, V, dtype="bf16", device="cuda", diag=False, diag_logits=False,
                 gemm_variant=FEF_GEMM_AUTO):
        self.B, self.K, self.block, self.d, self.V = B, K, block, d, V
        self.dtype = FEF_BF16 if dtype == "bf16" else FEF_F32
        self.torch_dtype = torch.bfloat16 if dtype == "bf16" else torch.float32
        self.device = torch.device(device)
        self.gemm_variant = gemm_variant
        dev = self.device
        self.out_tokens = torch.empty(B, K, dtype=torch.int32, device=dev)
        self.out_accept_len = torch.empty(B, dtype=torch.int32, device=dev)
        self.out_remask = torch.empty(B, block, dtype=torch.uint8, device=dev)
        self.diag = {}
        if diag:
            self.diag = {
                "draft_tokens": torch.empty(B, K, dtype=torch.int32, device=dev),
                "alpha": torch.empty(B, K, dtype=torch.float32, device=dev),
                "resid_mass": torch.empty(B, K, dtype=torch.float32, device=dev),
                "lse": torch.empty(2, B, K, dtype=torch.float32, device=dev),
                "conf_tok": torch.empty(B, K, dtype=torch.float32, device=dev),
            }
            if diag_logits:
                self.diag["logits"] = torch.empty(2, B, K, V, dtype=torch.float32, device=dev)
        p = self._params()
        nbytes = fef_workspace_bytes(p, K, block)
        if nbytes == 0:
            raise FefError(FEF_ERR_INVALID_ARG, fef_last_error())
        p.phase = FEF_PHASE_DRAFT          # split calls may pick another head kernel and layout
        nbytes = max(nbytes, fef_workspace_bytes(p, K, block))
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=dev)

    def _params(self, **kw):
        p = make_params(self.B, self.d, self.V, dtype=self.dtype, gemm_variant=self.gemm_variant, **kw)
        g = self.diag
        if g:
            p.diag_draft_tokens = g["draft_tokens"].data_ptr()
            p.diag_alpha = g["alpha"].data_ptr()
            p.diag_resid_mass = g["resid_mass"].data_ptr()
            p.diag_lse = g["lse"].data_ptr()
            p.diag_conf_tok = g["conf_tok"].data_ptr()
            if "logits" in g:
                p.diag_logits = g["logits"].data_ptr()
        return p

    def __call__(self, h_draft, h_target, W_vocab, seed, *, temperature=1.0, step=0, seq_base=0,
                 pos_base=0, n_rm=-1, final_pass=False, lowconf_scope=0, mask_in=None, pass_mask=None,
                 conf=None, draft_tokens=None, head_events=None, n_pass=0, seq_pass=None, seq_rounds=None,
                 tokens_state=None, phase=FEF_PHASE_FUSED, recorrupt_prob=1.0, greedy=False):
        for t, shape in ((h_draft, (self.B, self.K, self.d)), (h_target, (self.B, self.K, self.d)),
                         (W_vocab, (self.V, self.d))):
            if t is None:
                continue
            assert tuple(t.shape) == shape and t.dtype == self.torch_dtype and t.is_contiguous()
            assert t.device.type == "cuda"
        for t, dt, shape in ((mask_in, torch.uint8, (self.B, self.block)),
                             (pass_mask, torch.uint8, (self.B, self.block)),
                             (conf, torch.float32, (self.B, self.block)),
                             (draft_tokens, torch.int32, (self.B, self.K)),
                             (seq_pass, torch.int32, (self.B,)), (seq_rounds, torch.int32, (self.B,)),
                             (tokens_state, torch.int32, (self.B, self.block))):
            if t is not None:
                assert t.dtype == dt and tuple(t.shape) == shape and t.is_contiguous() and t.device.type == "cuda"
        p = self._params(temperature=temperature, step=step, seq_base=seq_base, pos_base=pos_base,
                         n_rm=n_rm, final_pass=final_pass, lowconf_scope=lowconf_scope)
        p.mask_in = None if mask_in is None else mask_in.data_ptr()
        p.pass_mask = None if pass_mask is None else pass_mask.data_ptr()
        p.conf = None if conf is None else conf.data_ptr()
        p.draft_tokens = None if draft_tokens is None else draft_tokens.data_ptr()
        p.phase = phase
        p.recorrupt_prob = recorrupt_prob
        p.greedy = int(greedy)
        p.n_pass = n_pass
        p.seq_pass = None if seq_pass is None else seq_pass.data_ptr()
        p.seq_rounds = None if seq_rounds is None else seq_rounds.data_ptr()
        p.tokens_state = None if tokens_state is None else tokens_state.data_ptr()
        p.workspace = self.workspace.data_ptr()
        p.workspace_bytes = self.workspace.numel()
        p.stream = torch.cuda.current_stream(self.device).cuda_stream
        if head_events is not None:     # pair of raw hipEvent_t handles (ints)
            p.ev_head_begin, p.ev_head_end = head_events
        fef_verify_step(p, h_draft, h_target, W_vocab, self.K, self.block, seed, self.out_tokens,
                        self.out_accept_len, self.out_remask)
        return self.out_tokens, self.out_accept_len, self.out_remask


def topn_step(vs, h, W_vocab, seed, n_transfer, *, temperature=1.0, step=0, seq_base=0, pos_base=0,
              mask_in=None, conf=None, tokens_state=None, greedy=False):
    """Baseline step (fef_topn_step) on the buffers of a VerifyStep of the same shape.  Returns
    (tokens [B,K], committed [B], remask [B,block])."""
    assert tuple(h.shape) == (vs.B, vs.K, vs.d) and h.dtype == vs.torch_dtype and h.is_contiguous()
    p = vs._params(temperature=temperature, step=step, seq_base=seq_base, pos_base=pos_base)
    p.mask_in = None if mask_in is None else mask_in.data_ptr()
    p.conf = None if conf is None else conf.data_ptr()
    p.tokens_state = None if tokens_state is None else tokens_state.data_ptr()
    p.greedy = int(greedy)
    p.workspace = vs.workspace.data_ptr()
    p.workspace_bytes = vs.workspace.numel()
    p.stream = torch.cuda.current_stream(vs.device).cuda_stream
    s = lib().fef_topn_step(ctypes.byref(p), _ptr(h), _ptr(W_vocab), vs.K, vs.block, ctypes.c_uint64(seed),
                            n_transfer, _ptr(vs.out_tokens), _ptr(vs.out_accept_len), _ptr(vs.out_remask))
    if s != FEF_OK:
        raise FefError(s, fef_last_error())
    return vs.out_tokens, vs.out_accept_len, vs.out_remask


class BlockDecoder:
    """Device-side state of Algorithm 2's outer loops for one block of B sequences: block mask,
    pass set, confidences, tokens, per-sequence pass and round counters.  `round()` enqueues one
    speculative round on top of that state and reads nothing back, so the rounds of a block can
    be queued back to back; a sequence that has finished its last pass is left untouched."""

    def __init__(self, step, n_pass, n_rm=-1, lowconf_scope=0, recorrupt_prob=1.0, greedy=False):
        self.vs, self.n_pass, self.n_rm, self.lowconf_scope = step, n_pass, n_rm, lowconf_scope
        self.recorrupt_prob, self.greedy = recorrupt_prob, greedy
        B, block, dev = step.B, step.block, step.device
        self.mask = torch.ones(B, block, dtype=torch.uint8, device=dev)
        self.pass_mask = torch.zeros(B, block, dtype=torch.uint8, device=dev)
        self.conf = torch.zeros(B, block, dtype=torch.float32, device=dev)
        self.tokens = torch.full((B, block), -1, dtype=torch.int32, device=dev)
        self.seq_pass = torch.zeros(B, dtype=torch.int32, device=dev)
        self.seq_rounds = torch.zeros(B, dtype=torch.int32, device=dev)

    def max_rounds(self):
        n_rm = self.vs.block // 2 if self.n_rm < 0 else min(self.n_rm, self.vs.block)
        return self.vs.block + (self.n_pass - 1) * max(n_rm, 1)

    def round(self, h_draft, h_target, W_vocab, seed, step, **kw):
        self.vs(h_draft, h_target, W_vocab, seed, step=step, n_rm=self.n_rm, lowconf_scope=self.lowconf_scope,
                recorrupt_prob=self.recorrupt_prob, greedy=self.greedy,
                mask_in=self.mask, pass_mask=self.pass_mask, conf=self.conf, n_pass=self.n_pass,
                seq_pass=self.seq_pass, seq_rounds=self.seq_rounds, tokens_state=self.tokens, **kw)
        # out_remask of this round is the mask of the next one (device-to-device, stream ordered)
        self.mask.copy_(self.vs.out_remask)
