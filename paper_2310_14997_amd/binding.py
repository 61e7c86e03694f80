"""Thin ctypes binding of libspcfg (include/spcfg.h).  Argument marshalling only.

PyTorch is used for device buffers and the stream handle; every step of the path runs in the library's
HIP kernels.  There is no CPU fallback: if the built library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspcfg.so")

PRECISION_FP32, PRECISION_BF16 = 0, 1
FLAG_ACCUMULATE_GRADS, FLAG_PER_SENTENCE_GRAMMAR, FLAG_FP32_MFMA, FLAG_BF16_SINGLE_FORWARD = 1, 2, 4, 8
PROF_CLASSES = 7


class SpcfgError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"libspcfg error {code}: {msg}")
        self.code = code


class Config(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("N", C.c_int32), ("P", C.c_int32), ("max_B", C.c_int32),
                ("max_n", C.c_int32), ("precision", C.c_int32), ("flags", C.c_uint32)]


_lib = None


def load():
    """Load libspcfg.so built in-tree (python -m paper_2310_14997_amd.build); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python paper_2310_14997_amd/build.py` "
                          "(there is no fallback path)")
    lib = C.CDLL(LIB_PATH)
    vp, sz, i32 = C.c_void_p, C.c_size_t, C.c_int32
    cfgp = C.POINTER(Config)
    lib.spcfg_workspace_bytes.argtypes = [cfgp, C.POINTER(sz)]
    lib.spcfg_workspace_bytes_for.argtypes = [cfgp, vp, i32, i32, C.POINTER(sz)]
    lib.spcfg_inside.argtypes = [cfgp, vp, vp, vp, vp, vp, i32, i32, vp, vp, sz, vp]
    lib.spcfg_inside_static.argtypes = [cfgp, vp, vp, vp, vp, vp, i32, i32, vp, vp]
    lib.spcfg_inside_backward.argtypes = [cfgp, vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.spcfg_inside_forward_backward.argtypes = [cfgp, vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp,
                                                  vp, sz, vp]
    lib.spcfg_rules_forward.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp]
    lib.spcfg_rules_backward.argtypes = [i32, i32, i32] + [vp] * 7 + [i32, i32] + [vp] * 10
    lib.spcfg_span_marginals.argtypes = [cfgp, vp, i32, i32, vp, sz, vp, vp, vp]
    lib.spcfg_mbr_decode_scratch_bytes.argtypes = [i32, i32, C.POINTER(sz)]
    lib.spcfg_mbr_decode.argtypes = [vp, vp, i32, i32, vp, vp, vp, sz, vp]
    lib.spcfg_rules_forward.restype = C.c_int
    lib.spcfg_rules_backward.restype = C.c_int
    lib.spcfg_strerror.argtypes = [C.c_int]
    lib.spcfg_strerror.restype = C.c_char_p
    lib.spcfg_last_hip_error.restype = C.c_char_p
    lib.spcfg_profile_enable.argtypes = [C.c_int]
    lib.spcfg_profile_read.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_int64), C.POINTER(C.c_double)]
    lib.spcfg_profile_class_name.argtypes = [C.c_int]
    lib.spcfg_profile_class_name.restype = C.c_char_p
    for name in ("spcfg_workspace_bytes", "spcfg_workspace_bytes_for", "spcfg_inside", "spcfg_inside_backward",
                 "spcfg_inside_forward_backward", "spcfg_inside_static", "spcfg_profile_enable", "spcfg_profile_read"):
        getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def _check(rc):
    if rc != 0:
        lib = load()
        msg = lib.spcfg_strerror(rc).decode()
        if rc == -6:
            msg += ": " + lib.spcfg_last_hip_error().decode()
        raise SpcfgError(rc, msg)


def make_config(N, P, max_B, max_n, precision=PRECISION_FP32, flags=0):
    return Config(C.sizeof(Config), int(N), int(P), int(max_B), int(max_n), int(precision), int(flags))


def _lengths_array(lengths):
    arr = np.ascontiguousarray(np.asarray(lengths, dtype=np.int32))
    return arr, arr.ctypes.data


def spcfg_workspace_bytes(cfg):
    out = C.c_size_t(0)
    _check(load().spcfg_workspace_bytes(C.byref(cfg), C.byref(out)))
    return out.value


def spcfg_workspace_bytes_for(cfg, lengths, n_max):
    arr, ptr = _lengths_array(lengths)
    out = C.c_size_t(0)
    _check(load().spcfg_workspace_bytes_for(C.byref(cfg), ptr, len(arr), int(n_max), C.byref(out)))
    return out.value


def _dev(t, name, shape=None):
    import torch
    if t is None:
        return None
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous() and t.dtype == torch.float32):
        raise TypeError(f"{name} must be a contiguous float32 device tensor")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} has shape {tuple(t.shape)}, expected {tuple(shape)}")
    return t.data_ptr()


def _stream():
    import torch
    return torch.cuda.current_stream().cuda_stream


def _ws(workspace):
    import torch
    if not (isinstance(workspace, torch.Tensor) and workspace.is_cuda and workspace.dtype == torch.uint8
            and workspace.is_contiguous()):
        raise TypeError("workspace must be a contiguous uint8 device tensor")
    return workspace.data_ptr(), workspace.numel()


def _grammar_shapes(cfg, L, B):
    """(N, M, shape of log_root, shape of L / R): per-sentence grammars carry a leading batch dimension."""
    N, M = L.shape[-2:]
    if cfg.flags & FLAG_PER_SENTENCE_GRAMMAR:
        return N, M, (B, N), (B, N, M)
    return N, M, (N,), (N, M)


def spcfg_inside(cfg, log_root, L, R, log_emit, lengths, logZ, workspace):
    """Enqueue the inside pass on torch's current stream; logZ [B] is written (see include/spcfg.h)."""
    B, n_max, P = log_emit.shape
    N, M, rs, gs = _grammar_shapes(cfg, L, B)
    arr, lptr = _lengths_array(lengths)
    wp, wb = _ws(workspace)
    _check(load().spcfg_inside(C.byref(cfg), _dev(log_root, "log_root", rs), _dev(L, "L", gs),
                               _dev(R, "R", gs), _dev(log_emit, "log_emit"), lptr, B, n_max,
                               _dev(logZ, "logZ", (B,)), wp, wb, _stream()))


STATIC_SCRATCH_BYTES = 64 << 20


def spcfg_inside_static(cfg, log_root, L, R, log_emit, lengths, logZ):
    """spcfg_inside with the workspace in the library's static device array: nothing is allocated (small batches only)."""
    B, n_max, P = log_emit.shape
    N, M, rs, gs = _grammar_shapes(cfg, L, B)
    arr, lptr = _lengths_array(lengths)
    _check(load().spcfg_inside_static(C.byref(cfg), _dev(log_root, "log_root", rs), _dev(L, "L", gs),
                                      _dev(R, "R", gs), _dev(log_emit, "log_emit"), lptr, B, n_max,
                                      _dev(logZ, "logZ", (B,)), _stream()))


def spcfg_inside_backward(cfg, log_root, L, R, log_emit, lengths, grad_logZ, grad_L, grad_R, grad_log_root,
                          grad_log_emit, workspace):
    """Enqueue the reverse pass; must follow spcfg_inside on the same inputs and workspace."""
    B, n_max, P = log_emit.shape
    N, M, rs, gs = _grammar_shapes(cfg, L, B)
    arr, lptr = _lengths_array(lengths)
    wp, wb = _ws(workspace)
    _check(load().spcfg_inside_backward(
        C.byref(cfg), _dev(log_root, "log_root", rs), _dev(L, "L", gs), _dev(R, "R", gs),
        _dev(log_emit, "log_emit"), lptr, B, n_max, _dev(grad_logZ, "grad_logZ", (B,)),
        _dev(grad_L, "grad_L", gs), _dev(grad_R, "grad_R", gs), _dev(grad_log_root, "grad_log_root", rs),
        _dev(grad_log_emit, "grad_log_emit", (B, n_max, P)), wp, wb, _stream()))


def spcfg_inside_forward_backward(cfg, log_root, L, R, log_emit, lengths, grad_logZ, logZ, grad_L, grad_R,
                                  grad_log_root, grad_log_emit, workspace):
    """Enqueue forward then reverse pass in one call."""
    B, n_max, P = log_emit.shape
    N, M, rs, gs = _grammar_shapes(cfg, L, B)
    arr, lptr = _lengths_array(lengths)
    wp, wb = _ws(workspace)
    _check(load().spcfg_inside_forward_backward(
        C.byref(cfg), _dev(log_root, "log_root", rs), _dev(L, "L", gs), _dev(R, "R", gs),
        _dev(log_emit, "log_emit"), lptr, B, n_max, _dev(grad_logZ, "grad_logZ", (B,)), _dev(logZ, "logZ", (B,)),
        _dev(grad_L, "grad_L", gs), _dev(grad_R, "grad_R", gs), _dev(grad_log_root, "grad_log_root", rs),
        _dev(grad_log_emit, "grad_log_emit", (B, n_max, P)), wp, wb, _stream()))


def _dev_i32(t, name, shape):
    import torch
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous() and t.dtype == torch.int32):
        raise TypeError(f"{name} must be a contiguous int32 device tensor")
    if tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} has shape {tuple(t.shape)}, expected {tuple(shape)}")
    return t.data_ptr()


def spcfg_rules_forward(root_logits, L_logits, R_logits, emis_logits, tokens, lengths, log_root, L, R, log_emit,
                        emis_lse):
    """Softmaxes of the rule scores and the per-token emission gather (see include/spcfg.h)."""
    N, M = L_logits.shape
    P, V = emis_logits.shape
    B, n_max = tokens.shape
    arr, lptr = _lengths_array(lengths)
    _check(load().spcfg_rules_forward(
        N, P, V, _dev(root_logits, "root_logits", (N,)), _dev(L_logits, "L_logits", (N, M)),
        _dev(R_logits, "R_logits", (N, M)), _dev(emis_logits, "emis_logits", (P, V)),
        _dev_i32(tokens, "tokens", (B, n_max)), lptr, B, n_max, _dev(log_root, "log_root", (N,)), _dev(L, "L", (N, M)),
        _dev(R, "R", (N, M)), _dev(log_emit, "log_emit", (B, n_max, P)), _dev(emis_lse, "emis_lse", (P,)), _stream()))


def spcfg_rules_backward(log_root, L, R, emis_logits, emis_lse, tokens, lengths, grad_log_root, grad_L, grad_R,
                         grad_log_emit, grad_root_logits, grad_L_logits, grad_R_logits, grad_emis_logits, scratch):
    """Backward of spcfg_rules_forward: gradients w.r.t. the four logit arrays."""
    N, M = L.shape
    P, V = emis_logits.shape
    B, n_max = tokens.shape
    arr, lptr = _lengths_array(lengths)
    _check(load().spcfg_rules_backward(
        N, P, V, _dev(log_root, "log_root", (N,)), _dev(L, "L", (N, M)), _dev(R, "R", (N, M)),
        _dev(emis_logits, "emis_logits", (P, V)), _dev(emis_lse, "emis_lse", (P,)),
        _dev_i32(tokens, "tokens", (B, n_max)), lptr, B, n_max, _dev(grad_log_root, "grad_log_root", (N,)),
        _dev(grad_L, "grad_L", (N, M)), _dev(grad_R, "grad_R", (N, M)),
        _dev(grad_log_emit, "grad_log_emit", (B, n_max, P)), _dev(grad_root_logits, "grad_root_logits", (N,)),
        _dev(grad_L_logits, "grad_L_logits", (N, M)), _dev(grad_R_logits, "grad_R_logits", (N, M)),
        _dev(grad_emis_logits, "grad_emis_logits", (P, V)), _dev(scratch, "scratch", (32, P)), _stream()))


def spcfg_span_marginals(cfg, lengths, n_max, workspace, span_post, span_label=None):
    """Span posteriors (and arg-max labels) from the workspace left by the forward + reverse pass."""
    arr, lptr = _lengths_array(lengths)
    B = len(arr)
    wp, wb = _ws(workspace)
    lab = None if span_label is None else _dev_i32(span_label, "span_label", (B, n_max, n_max))
    _check(load().spcfg_span_marginals(C.byref(cfg), lptr, B, int(n_max), wp, wb,
                                       _dev(span_post, "span_post", (B, n_max, n_max)), lab, _stream()))


def spcfg_mbr_decode_scratch_bytes(B, n_max):
    out = C.c_size_t(0)
    _check(load().spcfg_mbr_decode_scratch_bytes(int(B), int(n_max), C.byref(out)))
    return out.value


def spcfg_mbr_decode(span_post, lengths, tree_spans, tree_score, scratch):
    """Best bracketing per sentence under the span posteriors (see include/spcfg.h)."""
    arr, lptr = _lengths_array(lengths)
    B, n_max, _ = span_post.shape
    sp, sb = _ws(scratch)
    _check(load().spcfg_mbr_decode(_dev(span_post, "span_post", (B, n_max, n_max)), lptr, B, n_max,
                                   _dev_i32(tree_spans, "tree_spans", (B, n_max - 1, 2)),
                                   _dev(tree_score, "tree_score", (B,)), sp, sb, _stream()))


def spcfg_profile_enable(on):
    _check(load().spcfg_profile_enable(1 if on else 0))


def spcfg_profile_read():
    """Returns {class name: dict(ms, launches, work)} since profiling was enabled, and resets the counters."""
    lib = load()
    ms = (C.c_double * PROF_CLASSES)()
    ln = (C.c_int64 * PROF_CLASSES)()
    wk = (C.c_double * PROF_CLASSES)()
    _check(lib.spcfg_profile_read(ms, ln, wk))
    return {lib.spcfg_profile_class_name(c).decode(): dict(ms=ms[c], launches=ln[c], work=wk[c])
            for c in range(PROF_CLASSES)}


class Workload:
    """Device-resident buffers for one batch: a convenience holder used by the tests and the benchmark."""

    def __init__(self, inputs, precision=PRECISION_FP32, flags=0, device="cuda:0"):
        import torch
        self.torch = torch
        d = inputs
        self.B, self.N, self.P, self.n_max = d["B"], d["N"], d["P"], d["n_max"]
        self.lengths = np.ascontiguousarray(d["lengths"], dtype=np.int32)
        dev = torch.device(device)
        t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
        self.log_root, self.L, self.R, self.log_emit = t(d["log_root"]), t(d["L"]), t(d["R"]), t(d["log_emit"])
        if self.L.dim() == 3:  # one grammar per sentence
            flags |= FLAG_PER_SENTENCE_GRAMMAR
        self.cfg = make_config(self.N, self.P, self.B, self.n_max, precision, flags)
        nbytes = spcfg_workspace_bytes_for(self.cfg, self.lengths, self.n_max)
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        M = self.N + self.P
        f = dict(dtype=torch.float32, device=dev)
        self.logZ = torch.empty(self.B, **f)
        self.grad_L, self.grad_R = torch.empty_like(self.L), torch.empty_like(self.R)
        self.grad_log_root = torch.empty_like(self.log_root)
        self.grad_log_emit = torch.empty(self.B, self.n_max, self.P, **f)

    def forward(self):
        spcfg_inside(self.cfg, self.log_root, self.L, self.R, self.log_emit, self.lengths, self.logZ, self.workspace)
        return self.logZ

    def backward(self, grad_logZ=None):
        spcfg_inside_backward(self.cfg, self.log_root, self.L, self.R, self.log_emit, self.lengths, grad_logZ,
                              self.grad_L, self.grad_R, self.grad_log_root, self.grad_log_emit, self.workspace)

    def forward_backward(self, grad_logZ=None):
        spcfg_inside_forward_backward(self.cfg, self.log_root, self.L, self.R, self.log_emit, self.lengths,
                                      grad_logZ, self.logZ, self.grad_L, self.grad_R, self.grad_log_root,
                                      self.grad_log_emit, self.workspace)

    def span_marginals(self, with_labels=True):
        """Span posteriors [B, n_max, n_max] (and labels) of the last forward + backward."""
        torch = self.torch
        dev = self.logZ.device
        mu = torch.empty(self.B, self.n_max, self.n_max, dtype=torch.float32, device=dev)
        lab = torch.empty(self.B, self.n_max, self.n_max, dtype=torch.int32, device=dev) if with_labels else None
        spcfg_span_marginals(self.cfg, self.lengths, self.n_max, self.workspace, mu, lab)
        return mu, lab

    def mbr_decode(self, span_post):
        """(tree_spans [B, n_max-1, 2] int32, tree_score [B]) for the given span scores."""
        torch = self.torch
        dev = span_post.device
        spans = torch.empty(self.B, self.n_max - 1, 2, dtype=torch.int32, device=dev)
        score = torch.empty(self.B, dtype=torch.float32, device=dev)
        scratch = torch.empty(spcfg_mbr_decode_scratch_bytes(self.B, self.n_max), dtype=torch.uint8, device=dev)
        spcfg_mbr_decode(span_post, self.lengths, spans, score, scratch)
        return spans, score

    def results(self):
        self.torch.cuda.synchronize()
        g = lambda x: x.detach().cpu().numpy().astype(np.float64)
        return dict(logZ=g(self.logZ), grad_L=g(self.grad_L), grad_R=g(self.grad_R),
                    grad_log_root=g(self.grad_log_root), grad_log_emit=g(self.grad_log_emit))
