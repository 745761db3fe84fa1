"""ctypes binding of libhire.so: the same entry points as include/hire.h.

Argument marshalling only -- every step of the path runs in the library's HIP
kernels.  PyTorch supplies device memory and the current stream, nothing
else.  Importing this module fails if libhire.so has not been built
(`python -m paper_2402_09360_amd.build`); there is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("HIRE_LIB") or os.path.join(_HERE, "libhire.so")  # HIRE_LIB: e.g. the profiling build

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_2402_09360_amd.build` "
        "(hipcc, gfx950). The HiRE path has no fallback implementation.")

# torch is imported above on purpose: libhire.so must bind to the HIP runtime that PyTorch has already
# loaded (same SONAME), otherwise streams and launches would cross two runtimes.
_lib = C.CDLL(LIB_PATH)


def _hip_runtimes_loaded():
    try:
        with open("/proc/self/maps") as f:
            return sorted({line.split()[-1] for line in f if "libamdhip64" in line})
    except OSError:
        return []


if len(_hip_runtimes_loaded()) > 1:
    raise ImportError(
        "two HIP runtimes are loaded in this process (" + ", ".join(_hip_runtimes_loaded()) + "): libhire.so was "
        "opened before PyTorch. Import torch (or paper_2402_09360_amd.hire) before loading libhire.so directly.")

OK, EINVAL, ENOSPC, EUNSUPPORTED, ELAUNCH = 0, -1, -2, -3, -4
SCORER_INT4, SCORER_LOWRANK, SCORER_LRQ = 0, 1, 2
RELU, ORDER_RANK = 1, 2
MAX_BATCH = 64
MAX_RANK_ORDER_K = 4096


class _FFNLayer(C.Structure):
    _fields_ = [("d_model", C.c_int), ("d_ff", C.c_int), ("w1u", C.c_void_p), ("w2u", C.c_void_p),
                ("scorer_kind", C.c_int), ("q4", C.c_void_p), ("q4_scale", C.c_void_p), ("lr_a", C.c_void_p),
                ("lr_b", C.c_void_p), ("r", C.c_int), ("lr_a_scale", C.c_void_p), ("lr_b_scale", C.c_void_p),
                ("row_norm_bounds", C.c_void_p)]


class _SoftmaxLayer(C.Structure):
    _fields_ = [("d_model", C.c_int), ("vocab", C.c_int), ("w", C.c_void_p), ("scorer_kind", C.c_int),
                ("q4", C.c_void_p), ("q4_scale", C.c_void_p), ("lr_a", C.c_void_p), ("lr_b", C.c_void_p),
                ("r", C.c_int), ("lr_a_scale", C.c_void_p), ("lr_b_scale", C.c_void_p)]


_vp, _i, _sz = C.c_void_p, C.c_int, C.c_size_t
_lib.hire_version.restype = _i
_lib.hire_strerror.restype = C.c_char_p
_lib.hire_strerror.argtypes = [_i]
_lib.hire_last_launch_error.restype = C.c_char_p
_lib.hire_workspace_init.restype = _i
_lib.hire_workspace_init.argtypes = [_vp, _sz, _vp]
_lib.hire_debug_fast_fallbacks.restype = _i
_lib.hire_debug_fast_fallbacks.argtypes = [_vp, _vp, _vp]
_lib.hire_debug_fast_state.restype = _i
_lib.hire_debug_fast_state.argtypes = [_vp, _vp, _vp]
_lib.hire_debug_general_fallbacks.restype = _i
_lib.hire_debug_general_fallbacks.argtypes = [_vp, _vp, _vp]
_lib.hire_debug_plain_copy.restype = _i
_lib.hire_debug_plain_copy.argtypes = [_vp, _vp, _sz, _vp]
_lib.hire_set_scorer_clocks.restype = _i
_lib.hire_set_scorer_clocks.argtypes = [_vp, _sz]
_lib.hire_ffn_scorer_workgroups.restype = _i
_lib.hire_ffn_scorer_workgroups.argtypes = [_i]
_lib.hire_set_stage_events.restype = None
_lib.hire_set_stage_events.argtypes = [_vp]
_lib.hire_pack_int4_bytes.restype = _sz
_lib.hire_pack_int4_bytes.argtypes = [_i, _i]
_lib.hire_pack_int4.restype = _i
_lib.hire_pack_int4.argtypes = [_vp, _i, _i, _vp, _vp, _vp]
_lib.hire_unpack_int4.restype = _i
_lib.hire_unpack_int4.argtypes = [_vp, _i, _i, _vp, _vp]
_lib.hire_ffn_workspace_bytes.restype = _sz
_lib.hire_ffn_workspace_bytes.argtypes = [C.POINTER(_FFNLayer), _i, _i, _i]
_lib.hire_softmax_workspace_bytes.restype = _sz
_lib.hire_softmax_workspace_bytes.argtypes = [C.POINTER(_SoftmaxLayer), _i, _i, _i]
_lib.hire_topk_workspace_bytes.restype = _sz
_lib.hire_topk_workspace_bytes.argtypes = [_i, _i, _i, _i]
_lib.hire_ffn_step.restype = _i
_lib.hire_ffn_step.argtypes = [C.POINTER(_FFNLayer), _vp, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.hire_ffn_step_static.restype = _i
_lib.hire_ffn_step_static.argtypes = [C.POINTER(_FFNLayer), _vp, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
_lib.hire_ffn_group_workspace_bytes.restype = _sz
_lib.hire_ffn_group_workspace_bytes.argtypes = [C.POINTER(_FFNLayer), _i, _i, _i, _i]
_lib.hire_ffn_group_step.restype = _i
_lib.hire_ffn_group_step.argtypes = [C.POINTER(_FFNLayer), _vp, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz,
                                     _vp]
_lib.hire_ffn_shard_workspace_bytes.restype = _sz
_lib.hire_ffn_shard_workspace_bytes.argtypes = [C.POINTER(_FFNLayer), _i, _i, _i, _i]
_lib.hire_ffn_shard_step.restype = _i
_lib.hire_ffn_shard_step.argtypes = [C.POINTER(_FFNLayer), _vp, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz,
                                     _vp]
_lib.hire_ffn_commonpath_workspace_bytes.restype = _sz
_lib.hire_ffn_commonpath_workspace_bytes.argtypes = [C.POINTER(_FFNLayer), _i, _i, _i, _i, _i]
_lib.hire_ffn_commonpath_step.restype = _i
_lib.hire_ffn_commonpath_step.argtypes = [C.POINTER(_FFNLayer), _vp, _vp, _i, _vp, _i, _i, _i, _i, _vp, _vp, _vp, _vp,
                                          _vp, _vp, _vp, _sz, _vp]
_lib.hire_softmax_step.restype = _i
_lib.hire_softmax_step.argtypes = [C.POINTER(_SoftmaxLayer), _vp, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz,
                                   _vp]
_lib.topk_select.restype = _i
_lib.topk_select.argtypes = [_vp, _i, _i, _i, _i, _vp, _vp, _vp, _sz, _vp]


class HireError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        detail = f": {_lib.hire_last_launch_error().decode()}" if code == ELAUNCH else ""
        super().__init__(f"{where}: {_lib.hire_strerror(code).decode()} ({code}){detail}")


def _check(code: int, where: str):
    if code != OK:
        raise HireError(code, where)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def hire_version() -> int:
    return int(_lib.hire_version())


NUM_STAGE_EVENTS = 8
FFN_STAGES = ("quantise_x", "scorer", "select_kprime", "union", "gather_dot", "select_k", "second_layer")
FAST_FFN_STAGES = ("scorer", "select_gather", "select_w2", "reduce")   # batch 1, int4 scorer
SOFTMAX_STAGES = ("quantise_x", "scorer", "select_kprime", "union", "gather_dot", "select_k_softmax")


def hire_set_stage_events(events) -> None:
    """events: a ctypes array of NUM_STAGE_EVENTS hipEvent_t (see hiprt.Events.array), or None to switch off."""
    _lib.hire_set_stage_events(None if events is None else C.cast(events, C.c_void_p))


def hire_debug_fast_fallbacks(workspace: torch.Tensor, stream=None):
    out = (C.c_uint32 * 2)()
    _check(_lib.hire_debug_fast_fallbacks(_ptr(workspace), out, _stream(stream)), "hire_debug_fast_fallbacks")
    return int(out[0]), int(out[1])


def hire_force_exact_stage(on: bool) -> None:
    _lib.hire_force_exact_stage.restype = None
    _lib.hire_force_exact_stage.argtypes = [_i]
    _lib.hire_force_exact_stage(1 if on else 0)


def hire_debug_filter_stage(W: torch.Tensor, x: torch.Tensor, stream=None):
    """-> (stored [B, rows] float32, xnorm [B] float32, wnorm_max float, err_c float), see hire_debug.h."""
    _lib.hire_debug_filter_stage.restype = _i
    _lib.hire_debug_filter_stage.argtypes = [_vp, _vp, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp]
    rows, d = W.shape
    B = x.shape[0]
    dev = W.device
    n = torch.tensor([rows], dtype=torch.int32, device=dev)
    stored = torch.empty((B, rows), dtype=torch.float32, device=dev)
    xnorm = torch.zeros(B, dtype=torch.float32, device=dev)
    wmax = torch.zeros(1, dtype=torch.int32, device=dev)
    err_c = C.c_float(0.0)
    _check(_lib.hire_debug_filter_stage(_ptr(W), _ptr(x), B, d, rows, _ptr(n), _ptr(stored), _ptr(xnorm), _ptr(wmax),
                                        C.byref(err_c), _stream(stream)), "hire_debug_filter_stage")
    torch.cuda.synchronize()
    return stored, xnorm, float(wmax.view(torch.float32).item()), float(err_c.value)


def hire_debug_fast_state(workspace: torch.Tensor, stream=None):
    """(marker set, non-zero counters of the key histogram, counted activations) of a batch-1 FFN workspace."""
    out = (C.c_uint32 * 3)()
    _check(_lib.hire_debug_fast_state(_ptr(workspace), out, _stream(stream)), "hire_debug_fast_state")
    return tuple(int(v) for v in out)


def hire_debug_general_fallbacks(workspace: torch.Tensor, stream=None):
    out = (C.c_uint32 * 3)()
    _check(_lib.hire_debug_general_fallbacks(_ptr(workspace), out, _stream(stream)), "hire_debug_general_fallbacks")
    return tuple(int(v) for v in out)


def hire_debug_plain_copy(src: torch.Tensor, dst: torch.Tensor, stream=None) -> None:
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    _check(_lib.hire_debug_plain_copy(_ptr(src), _ptr(dst), nbytes, _stream(stream)), "hire_debug_plain_copy")


def hire_set_scorer_clocks(buf) -> None:
    """buf: uint64 device tensor with at least 2048 elements, or None."""
    if buf is None:
        _check(_lib.hire_set_scorer_clocks(None, 0), "hire_set_scorer_clocks")
    else:
        _check(_lib.hire_set_scorer_clocks(_ptr(buf), buf.numel() * buf.element_size()), "hire_set_scorer_clocks")


def hire_ffn_scorer_workgroups(d_ff: int) -> int:
    return int(_lib.hire_ffn_scorer_workgroups(d_ff))


def hire_force_generic_path(on: bool) -> None:
    _lib.hire_force_generic_path(1 if on else 0)


def hire_pack_int4_bytes(rows: int, cols: int) -> int:
    return int(_lib.hire_pack_int4_bytes(rows, cols))


def hire_pack_int4(w_bf16: torch.Tensor, stream=None):
    """int4 copy of a bf16 [rows, cols] device matrix: (packed uint8 blob, fp32 [rows] scales)."""
    assert w_bf16.is_cuda and w_bf16.dtype == torch.bfloat16 and w_bf16.is_contiguous() and w_bf16.dim() == 2
    rows, cols = w_bf16.shape
    nbytes = hire_pack_int4_bytes(rows, cols)
    if nbytes == 0:
        raise HireError(EINVAL, "hire_pack_int4_bytes")
    q4 = torch.empty(nbytes, dtype=torch.uint8, device=w_bf16.device)
    scale = torch.empty(rows, dtype=torch.float32, device=w_bf16.device)
    _check(_lib.hire_pack_int4(_ptr(w_bf16), rows, cols, _ptr(q4), _ptr(scale), _stream(stream)), "hire_pack_int4")
    return q4, scale


def hire_unpack_int4(q4: torch.Tensor, rows: int, cols: int, stream=None) -> torch.Tensor:
    codes = torch.empty((rows, cols), dtype=torch.int8, device=q4.device)
    _check(_lib.hire_unpack_int4(_ptr(q4), rows, cols, _ptr(codes), _stream(stream)), "hire_unpack_int4")
    return codes


def pack_lrq(z1: torch.Tensor, z2: torch.Tensor):
    """int4 copies for HiRE-LRQ of the low-rank factors z1 bf16 [d_model, r] (packed transposed, one scale per column
    of z1) and z2 bf16 [rows, r]: (blob1, scales1 [r], blob2, scales2 [rows])."""
    q1, s1 = hire_pack_int4(z1.t().contiguous())
    q2, s2 = hire_pack_int4(z2.contiguous())
    return q1, s1, q2, s2


class FFNLayer:
    """Device tensors of one FFN layer plus the C descriptor that points at them."""

    def __init__(self, w1u, w2u, q4=None, q4_scale=None, lr_a=None, lr_b=None, lrq=None, prepare=True):
        """lrq: (int4 blob of Z1 transposed, its scales [r], int4 blob of Z2, its scales [d_ff]) for HiRE-LRQ.
        prepare: run hire_lr_prepare for a low-rank layer (False: its batch-1 steps take the general sequence)."""
        for t in (w1u, w2u):
            assert t.is_cuda and t.dtype == torch.bfloat16 and t.is_contiguous()
        self.w1u, self.w2u, self.q4, self.q4_scale, self.lr_a, self.lr_b = w1u, w2u, q4, q4_scale, lr_a, lr_b
        self.d_ff, self.d_model = w1u.shape
        self.kind = SCORER_LOWRANK if lr_a is not None else SCORER_INT4
        self.r = int(lr_a.shape[1]) if lr_a is not None else 0
        self.lr_a_scale = self.lr_b_scale = None
        if lrq is not None:
            self.lr_a, self.lr_a_scale, self.lr_b, self.lr_b_scale = lrq
            self.kind, self.r = SCORER_LRQ, int(self.lr_a_scale.numel())
        p = lambda t: t.data_ptr() if t is not None else None
        self.c = _FFNLayer(self.d_model, self.d_ff, w1u.data_ptr(), w2u.data_ptr(), self.kind, p(q4), p(q4_scale),
                           p(self.lr_a), p(self.lr_b), self.r, p(self.lr_a_scale), p(self.lr_b_scale), None)
        self.row_norm_bounds = None
        if self.kind in (SCORER_LOWRANK, SCORER_LRQ) and prepare:
            # one-off preparation: row-norm bounds that let batch-1 steps take the short kernel sequence
            self.row_norm_bounds = torch.zeros(2, dtype=torch.float32, device=w1u.device)
            _lib.hire_lr_prepare.restype = _i
            _lib.hire_lr_prepare.argtypes = [C.c_void_p, _vp, _vp]
            _check(_lib.hire_lr_prepare(C.byref(self.c), _ptr(self.row_norm_bounds), _stream(None)), "hire_lr_prepare")
            torch.cuda.synchronize()
            self.c.row_norm_bounds = self.row_norm_bounds.data_ptr()

    @classmethod
    def with_lrq_scorer(cls, w1u, w2u, z1, z2):
        """HiRE-LRQ: z1 bf16 [d_model, r], z2 bf16 [d_ff, r]; both are quantised to int4 row by row (z1 transposed)."""
        return cls(w1u, w2u, lrq=pack_lrq(z1, z2))

    @classmethod
    def with_int4_scorer(cls, w1u, w2u):
        q4, s = hire_pack_int4(w1u)
        return cls(w1u, w2u, q4=q4, q4_scale=s)


class SoftmaxLayer:
    def __init__(self, w, q4=None, q4_scale=None, lr_a=None, lr_b=None, lrq=None):
        assert w.is_cuda and w.dtype == torch.bfloat16 and w.is_contiguous()
        self.w, self.q4, self.q4_scale, self.lr_a, self.lr_b = w, q4, q4_scale, lr_a, lr_b
        self.vocab, self.d_model = w.shape
        self.kind = SCORER_LOWRANK if lr_a is not None else SCORER_INT4
        self.r = int(lr_a.shape[1]) if lr_a is not None else 0
        self.lr_a_scale = self.lr_b_scale = None
        if lrq is not None:
            self.lr_a, self.lr_a_scale, self.lr_b, self.lr_b_scale = lrq
            self.kind, self.r = SCORER_LRQ, int(self.lr_a_scale.numel())
        p = lambda t: t.data_ptr() if t is not None else None
        self.c = _SoftmaxLayer(self.d_model, self.vocab, w.data_ptr(), self.kind, p(q4), p(q4_scale), p(self.lr_a),
                               p(self.lr_b), self.r, p(self.lr_a_scale), p(self.lr_b_scale))

    @classmethod
    def with_lrq_scorer(cls, w, z1, z2):
        return cls(w, lrq=pack_lrq(z1, z2))

    @classmethod
    def with_int4_scorer(cls, w):
        q4, s = hire_pack_int4(w)
        return cls(w, q4=q4, q4_scale=s)


def hire_ffn_workspace_bytes(layer: FFNLayer, B: int, k: int, kprime: int) -> int:
    return int(_lib.hire_ffn_workspace_bytes(C.byref(layer.c), B, k, kprime))


def hire_softmax_workspace_bytes(layer: SoftmaxLayer, B: int, k: int, kprime: int) -> int:
    return int(_lib.hire_softmax_workspace_bytes(C.byref(layer.c), B, k, kprime))


def hire_topk_workspace_bytes(B: int, N: int, k: int, flags: int = 0) -> int:
    return int(_lib.hire_topk_workspace_bytes(B, N, k, flags))


def alloc_workspace(nbytes: int, device="cuda") -> torch.Tensor:
    if nbytes <= 0:
        raise HireError(EINVAL, "workspace size")
    ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
    _check(_lib.hire_workspace_init(_ptr(ws), ws.numel(), _stream(None)), "hire_workspace_init")
    return ws


class FFNOutputs:
    """Caller-owned output buffers of hire_ffn_step (allocate once, reuse every step)."""

    def __init__(self, layer: FFNLayer, B: int, k: int, kprime: int, debug: bool = False):
        dev = layer.w1u.device
        self.y = torch.empty((B, layer.d_model), dtype=torch.float32, device=dev)
        self.topk_idx = torch.empty((B, k), dtype=torch.int32, device=dev)
        self.topk_val = torch.empty((B, k), dtype=torch.float32, device=dev)
        self.cand_idx = torch.empty(min(B * kprime, layer.d_ff), dtype=torch.int32, device=dev)
        self.n_cand = torch.zeros(1, dtype=torch.int32, device=dev)
        self.scorer_acc = (torch.empty((B, layer.d_ff), dtype=torch.int32, device=dev)
                           if debug and layer.kind == SCORER_INT4 else None)


def hire_ffn_step(layer: FFNLayer, x: torch.Tensor, k: int, kprime: int, out: FFNOutputs, workspace: torch.Tensor,
                  stream=None, minimal: bool = False) -> None:
    """Enqueue one HiRE-FFN step.  With minimal=True only y is requested (the optional outputs are skipped)."""
    B = x.shape[0]
    opt = (None,) * 5 if minimal else (out.topk_idx, out.topk_val, out.cand_idx, out.n_cand, out.scorer_acc)
    rc = _lib.hire_ffn_step(C.byref(layer.c), _ptr(x), B, k, kprime, _ptr(out.y), *[_ptr(t) for t in opt],
                            _ptr(workspace), workspace.numel(), _stream(stream))
    _check(rc, "hire_ffn_step")


STATIC_SCRATCH_BYTES = 8 << 20


def hire_ffn_step_static(layer: FFNLayer, x: torch.Tensor, k: int, kprime: int, out: FFNOutputs, stream=None,
                         minimal: bool = False) -> None:
    """hire_ffn_step on the library's own statically allocated scratch memory: no workspace argument, nothing
    allocated by the call (for callers that cannot allocate; steps beyond STATIC_SCRATCH_BYTES are refused)."""
    B = x.shape[0]
    opt = (None,) * 5 if minimal else (out.topk_idx, out.topk_val, out.cand_idx, out.n_cand, out.scorer_acc)
    rc = _lib.hire_ffn_step_static(C.byref(layer.c), _ptr(x), B, k, kprime, _ptr(out.y), *[_ptr(t) for t in opt],
                                   _stream(stream))
    _check(rc, "hire_ffn_step_static")


def hire_ffn_group_workspace_bytes(layer: FFNLayer, B: int, k: int, kprime: int, group: int) -> int:
    return int(_lib.hire_ffn_group_workspace_bytes(C.byref(layer.c), B, k, kprime, group))


class FFNGroupOutputs:
    """Caller-owned output buffers of hire_ffn_group_step."""

    def __init__(self, layer: FFNLayer, B: int, k: int, kprime: int, group: int, debug: bool = False):
        dev = layer.w1u.device
        self.y = torch.empty((B, layer.d_model), dtype=torch.float32, device=dev)
        self.topk_group = torch.empty((B, k // group), dtype=torch.int32, device=dev)
        self.topk_val = torch.empty((B, k), dtype=torch.float32, device=dev)
        self.cand_group = torch.empty(min(B * (kprime // group), layer.d_ff // group), dtype=torch.int32, device=dev)
        self.n_cand = torch.zeros(1, dtype=torch.int32, device=dev)
        self.scorer_acc = (torch.empty((B, layer.d_ff), dtype=torch.int32, device=dev)
                           if debug and layer.kind == SCORER_INT4 else None)


def hire_ffn_group_step(layer: FFNLayer, x: torch.Tensor, k: int, kprime: int, group: int, out: FFNGroupOutputs,
                        workspace: torch.Tensor, stream=None, minimal: bool = False) -> None:
    """Enqueue one group-sparse HiRE-FFN step.  With minimal=True only y is requested."""
    B = x.shape[0]
    opt = (None,) * 5 if minimal else (out.topk_group, out.topk_val, out.cand_group, out.n_cand, out.scorer_acc)
    rc = _lib.hire_ffn_group_step(C.byref(layer.c), _ptr(x), B, k, kprime, group, _ptr(out.y),
                                  *[_ptr(t) for t in opt], _ptr(workspace), workspace.numel(), _stream(stream))
    _check(rc, "hire_ffn_group_step")


def hire_ffn_commonpath_workspace_bytes(layer: FFNLayer, m1: int, B: int, k: int, kprime: int, group: int) -> int:
    return int(_lib.hire_ffn_commonpath_workspace_bytes(C.byref(layer.c), m1, B, k, kprime, group))


def hire_ffn_commonpath_step(layer: FFNLayer, dense_w1u, dense_w2u, x: torch.Tensor, k: int, kprime: int, group: int,
                             out: "FFNGroupOutputs", workspace: torch.Tensor, stream=None,
                             minimal: bool = False) -> None:
    """Enqueue one CommonPath FFN step: dense units (bf16 [m1, d] tensors, or None for m1 = 0) plus the
    group-sparse step on `layer`.  Outputs as for hire_ffn_group_step."""
    B = x.shape[0]
    m1 = 0 if dense_w1u is None else dense_w1u.shape[0]
    opt = (None,) * 5 if minimal else (out.topk_group, out.topk_val, out.cand_group, out.n_cand, out.scorer_acc)
    rc = _lib.hire_ffn_commonpath_step(C.byref(layer.c), _ptr(dense_w1u), _ptr(dense_w2u), m1, _ptr(x), B, k, kprime,
                                       group, _ptr(out.y), *[_ptr(t) for t in opt], _ptr(workspace),
                                       workspace.numel(), _stream(stream))
    _check(rc, "hire_ffn_commonpath_step")


def hire_ffn_shard_workspace_bytes(layer: FFNLayer, B: int, k: int, kprime: int, shards: int) -> int:
    return int(_lib.hire_ffn_shard_workspace_bytes(C.byref(layer.c), B, k, kprime, shards))


class FFNShardOutputs:
    """Caller-owned output buffers of hire_ffn_shard_step."""

    def __init__(self, layer: FFNLayer, B: int, k: int, kprime: int, shards: int, debug: bool = False):
        dev = layer.w1u.device
        qp, q = -(-kprime // shards), -(-k // shards)  # quotas that do not divide are rounded up (Algorithm 2)
        cap = min(B * qp, layer.d_ff // shards)
        self.y = torch.empty((B, layer.d_model), dtype=torch.float32, device=dev)
        self.topk_idx = torch.empty((B, shards * q), dtype=torch.int32, device=dev)
        self.topk_val = torch.empty((B, shards * q), dtype=torch.float32, device=dev)
        self.cand_idx = torch.zeros((shards, cap), dtype=torch.int32, device=dev)
        self.n_cand = torch.zeros(shards, dtype=torch.int32, device=dev)
        self.scorer_acc = torch.empty((B, layer.d_ff), dtype=torch.int32, device=dev) if debug else None


def hire_ffn_shard_step(layer: FFNLayer, x: torch.Tensor, k: int, kprime: int, shards: int, out: FFNShardOutputs,
                        workspace: torch.Tensor, stream=None, minimal: bool = False) -> None:
    """Enqueue one HiRE-FFN step with Algorithm 2's sharded top-k.  With minimal=True only y is requested."""
    B = x.shape[0]
    opt = (None,) * 5 if minimal else (out.topk_idx, out.topk_val, out.cand_idx, out.n_cand, out.scorer_acc)
    rc = _lib.hire_ffn_shard_step(C.byref(layer.c), _ptr(x), B, k, kprime, shards, _ptr(out.y),
                                  *[_ptr(t) for t in opt], _ptr(workspace), workspace.numel(), _stream(stream))
    _check(rc, "hire_ffn_shard_step")


class SoftmaxOutputs:
    def __init__(self, layer: SoftmaxLayer, B: int, k: int, kprime: int, debug: bool = False):
        dev = layer.w.device
        self.top_idx = torch.empty((B, k), dtype=torch.int32, device=dev)
        self.top_prob = torch.empty((B, k), dtype=torch.float32, device=dev)
        self.top_logit = torch.empty((B, k), dtype=torch.float32, device=dev)
        self.cand_idx = torch.empty(min(B * kprime, layer.vocab), dtype=torch.int32, device=dev)
        self.n_cand = torch.zeros(1, dtype=torch.int32, device=dev)
        self.scorer_acc = (torch.empty((B, layer.vocab), dtype=torch.int32, device=dev)
                           if debug and layer.kind == SCORER_INT4 else None)


def hire_softmax_step(layer: SoftmaxLayer, x: torch.Tensor, k: int, kprime: int, out: SoftmaxOutputs,
                      workspace: torch.Tensor, stream=None, minimal: bool = False) -> None:
    B = x.shape[0]
    opt = (None,) * 4 if minimal else (out.top_logit, out.cand_idx, out.n_cand, out.scorer_acc)
    rc = _lib.hire_softmax_step(C.byref(layer.c), _ptr(x), B, k, kprime, _ptr(out.top_idx), _ptr(out.top_prob),
                                *[_ptr(t) for t in opt], _ptr(workspace), workspace.numel(), _stream(stream))
    _check(rc, "hire_softmax_step")


def topk_select(scores: torch.Tensor, k: int, relu: bool = False, rank_order: bool = False, want_values: bool = True,
                stream=None, workspace: torch.Tensor | None = None):
    """Indices (int32 [B,k]) and values (fp32 [B,k]) of the k largest entries of each row of scores fp32 [B,N].
    workspace: one from alloc_workspace(hire_topk_workspace_bytes(...)) to reuse over calls of the same shape (long
    rows then select through its histograms from the second call on); a fresh one is made otherwise."""
    assert scores.is_cuda and scores.dtype == torch.float32 and scores.is_contiguous() and scores.dim() == 2
    B, N = scores.shape
    flags = (RELU if relu else 0) | (ORDER_RANK if rank_order else 0)
    idx = torch.empty((B, max(k, 0)), dtype=torch.int32, device=scores.device)
    val = torch.empty((B, max(k, 0)), dtype=torch.float32, device=scores.device) if want_values else None
    ws = workspace if workspace is not None else alloc_workspace(max(hire_topk_workspace_bytes(B, N, k, flags), 256),
                                                                 scores.device)
    _check(_lib.topk_select(_ptr(scores), B, N, k, flags, _ptr(idx), _ptr(val), _ptr(ws), ws.numel(), _stream(stream)),
           "topk_select")
    return idx, val


def bf16_from_bits(bits, device="cuda") -> torch.Tensor:
    """numpy uint16 bf16 bit patterns -> torch.bfloat16 tensor on the device (a copy of the same bytes)."""
    import numpy as np
    a = np.ascontiguousarray(bits, dtype=np.uint16)
    return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).to(device)
