"""ctypes binding over libhybridattn.so (include/hybrid_attn.h).

Argument marshalling only: every step of the forward runs in the HIP kernels of the library.
PyTorch supplies device memory and the current HIP stream.  There is no CPU fallback; if the
library is not built, or no GPU is present, calls raise.
"""
from __future__ import annotations

import contextlib
import ctypes
import functools
import inspect
import os
from dataclasses import dataclass
from typing import Optional

import torch  # imported before the library so that both share torch's HIP runtime

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("HYBRID_ATTN_LIB", os.path.join(_HERE, "lib", "libhybridattn.so"))

HA_OK, HA_ERR_NULL, HA_ERR_SHAPE, HA_ERR_UNSUPPORTED, HA_ERR_ALIGN, HA_ERR_WORKSPACE, HA_ERR_DEVICE, HA_ERR_INFEASIBLE = range(8)
HA_BF16, HA_F32 = 0, 1
HA_ACT_SOFTMAX, HA_ACT_EXP, HA_ACT_RELU = 0, 1, 2


class ha_feature_map(ctypes.Structure):
    _fields_ = [("w1", ctypes.c_void_p), ("b1", ctypes.c_void_p), ("w2", ctypes.c_void_p), ("b2", ctypes.c_void_p),
                ("d_hidden", ctypes.c_int32), ("d_out", ctypes.c_int32), ("poly_degree", ctypes.c_int32),
                ("out_act", ctypes.c_int32),
                ("w_mid", ctypes.c_void_p), ("b_mid", ctypes.c_void_p), ("d_mid", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class ha_feature_map_grad(ctypes.Structure):
    _fields_ = [("w1", ctypes.c_void_p), ("b1", ctypes.c_void_p), ("w2", ctypes.c_void_p), ("b2", ctypes.c_void_p),
                ("w_mid", ctypes.c_void_p), ("b_mid", ctypes.c_void_p)]


class ha_optimizer(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("step", ctypes.c_int32), ("lr", ctypes.c_float), ("grad_scale", ctypes.c_float),
                ("beta1", ctypes.c_float), ("beta2", ctypes.c_float), ("eps", ctypes.c_float), ("weight_decay", ctypes.c_float)]


HA_OPT_SGD, HA_OPT_ADAMW = 0, 1


class ha_problem(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("N", ctypes.c_int32), ("d_head", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("block_size", ctypes.c_int32), ("hybrid_rate", ctypes.c_int32),
                ("softmax_scale", ctypes.c_float),
                ("stride_b", ctypes.c_int64), ("stride_h", ctypes.c_int64), ("stride_n", ctypes.c_int64),
                ("split_granularity", ctypes.c_int32), ("causal_chunk", ctypes.c_int32),
                ("local_window", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class HybridAttnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        lib = _lib()
        msg = lib.hybrid_attn_status_string(status).decode()
        if status == HA_ERR_DEVICE:
            msg += f" [hipError {lib.hybrid_attn_last_device_error()}]"
        super().__init__(f"{where}: {msg} (status {status})")


_LIB = None


def _lib():
    """Load the shared library once.  Raises if it has not been built (no fallback)."""
    global _LIB
    if _LIB is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2509_24899_amd.build` "
                               "(or __graft_entry__.build()) first; there is no CPU fallback")
        lib = ctypes.CDLL(LIB_PATH)
        P, FM = ctypes.POINTER(ha_problem), ctypes.POINTER(ha_feature_map)
        vp = ctypes.c_void_p
        lib.hybrid_attn_validate.argtypes = [P, FM, FM]
        lib.hybrid_attn_validate.restype = ctypes.c_int
        lib.hybrid_attn_workspace_bytes.argtypes = [P, FM, FM]
        lib.hybrid_attn_workspace_bytes.restype = ctypes.c_size_t
        lib.hybrid_attn_forward.argtypes = [P, vp, vp, vp, FM, FM, vp, vp, ctypes.c_size_t, vp]
        lib.hybrid_attn_forward.restype = ctypes.c_int
        lib.hybrid_attn_forward_static.argtypes = [P, vp, vp, vp, FM, FM, vp, vp]
        lib.hybrid_attn_forward_static.restype = ctypes.c_int
        lib.hybrid_attn_static_scratch_bytes.argtypes = []
        lib.hybrid_attn_static_scratch_bytes.restype = ctypes.c_size_t
        lib.hybrid_attn_linear_state.argtypes = [P, vp, vp, FM, vp, vp, vp, ctypes.c_size_t, vp]
        lib.hybrid_attn_linear_state.restype = ctypes.c_int
        lib.hybrid_attn_status_string.argtypes = [ctypes.c_int]
        lib.hybrid_attn_status_string.restype = ctypes.c_char_p
        lib.hybrid_attn_last_device_error.argtypes = []
        lib.hybrid_attn_last_device_error.restype = ctypes.c_int
        lib.hybrid_attn_profile_enable.argtypes = [ctypes.c_int]
        lib.hybrid_attn_profile_enable.restype = ctypes.c_int
        lib.hybrid_attn_profile_read.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_float)]
        lib.hybrid_attn_profile_read.restype = ctypes.c_int
        lib.hybrid_attn_profile_count.argtypes = []
        lib.hybrid_attn_profile_count.restype = ctypes.c_int
        lib.hybrid_attn_mfma_probe.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t,
                                               ctypes.POINTER(ctypes.c_double), ctypes.c_void_p]
        lib.hybrid_attn_mfma_probe.restype = ctypes.c_int
        dp = ctypes.POINTER(ctypes.c_double)
        lib.hybrid_attn_value_distill_workspace_bytes.argtypes = [P, FM, FM]
        lib.hybrid_attn_value_distill_workspace_bytes.restype = ctypes.c_size_t
        lib.hybrid_attn_value_distill_loss.argtypes = [P, vp, vp, vp, FM, FM, ctypes.c_int, vp, vp, vp, vp,
                                                       ctypes.c_size_t, vp]
        lib.hybrid_attn_value_distill_loss.restype = ctypes.c_int
        lib.hybrid_attn_select_rates.argtypes = [ctypes.c_int, ctypes.c_int, dp, dp, ctypes.c_double,
                                                 ctypes.POINTER(ctypes.c_int), dp, dp]
        lib.hybrid_attn_select_rates.restype = ctypes.c_int
        lib.hybrid_attn_value_distill_grad_workspace_bytes.argtypes = [P, FM, FM]
        lib.hybrid_attn_value_distill_grad_workspace_bytes.restype = ctypes.c_size_t
        FMG = ctypes.POINTER(ha_feature_map_grad)
        lib.hybrid_attn_value_distill_grad.argtypes = [P, vp, vp, vp, FM, FM, ctypes.c_int, ctypes.c_int, vp, vp, vp, vp,
                                                       FMG, FMG, vp, ctypes.c_size_t, vp]
        lib.hybrid_attn_value_distill_grad.restype = ctypes.c_int
        lib.hybrid_attn_param_update.argtypes = [ctypes.POINTER(ha_optimizer), ctypes.c_size_t, vp, vp, vp, vp, vp,
                                                 ctypes.c_int32, vp]
        lib.hybrid_attn_param_update.restype = ctypes.c_int
        lib.hybrid_attn_abi_version.argtypes = []
        lib.hybrid_attn_abi_version.restype = ctypes.c_int
        _LIB = lib
    return _LIB


@dataclass
class FeatureMap:
    """Device tensors of one feature map: w1 [H, Hd, d], b1 [H, Hd] fp32 or None, w2 [H, F, Hd],
    b2 [H, F] fp32 or None; weights in the io dtype of q, k, v.  Three-layer map: w_mid [H, Dm, Hd],
    b_mid [H, Dm] fp32 or None, and w2 is [H, F, Dm]."""
    w1: torch.Tensor
    b1: Optional[torch.Tensor]
    w2: torch.Tensor
    b2: Optional[torch.Tensor]
    poly_degree: int = 2
    out_act: int = HA_ACT_SOFTMAX
    w_mid: Optional[torch.Tensor] = None
    b_mid: Optional[torch.Tensor] = None

    def check(self, H: int, d_head: int, dtype, device) -> None:
        """The C ABI reads these tensors through raw pointers with the shapes and dtype it derives from the problem;
        a mismatch would be garbage or an out-of-bounds device read, so every dimension, dtype and device is checked
        here against the problem's (H heads of width d_head, io dtype, device of q)."""
        def need(cond, what):
            if not cond:
                raise ValueError(f"feature map does not match the problem: {what}")
        Hd = self.w1.shape[1] if self.w1.dim() == 3 else -1
        need(self.w1.dim() == 3 and tuple(self.w1.shape) == (H, Hd, d_head), f"w1 must be [H={H}, d_hidden, d_head={d_head}], got {tuple(self.w1.shape)}")
        kl = Hd
        if self.w_mid is not None:
            need(self.w_mid.dim() == 3 and tuple(self.w_mid.shape[::2]) == (H, Hd), f"w_mid must be [H={H}, d_mid, d_hidden={Hd}], got {tuple(self.w_mid.shape)}")
            kl = self.w_mid.shape[1]
        need(self.w2.dim() == 3 and self.w2.shape[0] == H and self.w2.shape[2] == kl, f"w2 must be [H={H}, d_out, {kl}], got {tuple(self.w2.shape)}")
        F = self.w2.shape[1]
        for name, b, width in (("b1", self.b1, Hd), ("b2", self.b2, F), ("b_mid", self.b_mid, kl)):
            if b is not None:
                need(name != "b_mid" or self.w_mid is not None, "b_mid given without w_mid")
                need(tuple(b.shape) == (H, width), f"{name} must be [H={H}, {width}], got {tuple(b.shape)}")
                need(b.device == device, f"{name} is on {b.device}, q on {device}")
        for name, t in (("w1", self.w1), ("w2", self.w2), ("w_mid", self.w_mid)):
            if t is not None:
                need(t.dtype == dtype, f"{name} is {t.dtype}, q is {dtype}")
                need(t.device == device, f"{name} is on {t.device}, q on {device}")
        need(self.poly_degree >= 1 and F % self.poly_degree == 0, f"poly_degree {self.poly_degree} must divide d_out {F}")

    def c_struct(self) -> ha_feature_map:
        for t in (self.w1, self.w2, self.w_mid):
            if t is not None and not t.is_contiguous():
                raise ValueError("feature-map weights must be contiguous")
        for b in (self.b1, self.b2, self.b_mid):
            if b is not None and (b.dtype != torch.float32 or not b.is_contiguous()):
                raise ValueError("feature-map biases must be contiguous fp32")
        return ha_feature_map(self.w1.data_ptr(), self.b1.data_ptr() if self.b1 is not None else None,
                              self.w2.data_ptr(), self.b2.data_ptr() if self.b2 is not None else None,
                              self.w1.shape[1], self.w2.shape[1], self.poly_degree, self.out_act,
                              self.w_mid.data_ptr() if self.w_mid is not None else None,
                              self.b_mid.data_ptr() if self.b_mid is not None else None,
                              self.w_mid.shape[1] if self.w_mid is not None else 0, 0)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return HA_BF16
    if t.dtype == torch.float32:
        return HA_F32
    raise ValueError(f"unsupported dtype {t.dtype}: q, k, v must be bfloat16 or float32")


def make_problem(q: torch.Tensor, hybrid_rate, block_size: int, softmax_scale: float) -> ha_problem:
    """ha_problem for a [B, H, N, d] tensor view (any strides with a contiguous last dim).  hybrid_rate: R, or a pair
    (R, g) for the block-granular variant of the split (groups of g tokens, every R-th group softmax tokens), or a
    triple (R, g, C) for the chunk-causal variant on top (chunks of C tokens; g = 0 for the per-token split), or
    (0, 0, 0, W) for the local-window variant (W tokens on either side of the query's tile)."""
    granularity, causal, window = 0, 0, 0
    if isinstance(hybrid_rate, (tuple, list)):
        if len(hybrid_rate) == 4:
            hybrid_rate, granularity, causal, window = hybrid_rate
        elif len(hybrid_rate) == 3:
            hybrid_rate, granularity, causal = hybrid_rate
        else:
            hybrid_rate, granularity = hybrid_rate
    if q.dim() != 4 or q.stride(3) != 1:
        raise ValueError("q, k, v must be [B, H, N, d] views with a contiguous last dimension")
    B, H, N, d = q.shape
    return ha_problem(B, H, N, d, _dtype_code(q), block_size, hybrid_rate, softmax_scale,
                      q.stride(0), q.stride(1), q.stride(2), int(granularity), int(causal), int(window), 0)


def _fm_ptr(fm, like=None):
    """(struct, pointer) of a feature map for the C ABI; with `like` (the q or k tensor of the call) a FeatureMap is
    first checked against its heads, head width, dtype and device."""
    if fm is None:
        return None, None
    if isinstance(fm, FeatureMap) and like is not None:
        fm.check(like.shape[1], like.shape[3], like.dtype, like.device)
    s = fm.c_struct() if isinstance(fm, FeatureMap) else fm
    return s, ctypes.byref(s)


def _allocations_follow_stream(fn):
    """Runs `fn` with its `stream` argument (if given) as torch's current stream, see _alloc_on."""
    sig = inspect.signature(fn)

    @functools.wraps(fn)
    def wrapper(*args, **kwargs):
        with _alloc_on(sig.bind(*args, **kwargs).arguments.get("stream")):
            return fn(*args, **kwargs)
    return wrapper


def _alloc_on(stream):
    """Context for the binding's own allocations: with an explicit stream they are made under it, so that torch's
    caching allocator ties the block to the stream the kernels run on (a block allocated under another stream could be
    handed out again while they still run)."""
    return torch.cuda.stream(stream) if stream is not None else contextlib.nullcontext()


def hybrid_attn_validate(problem: ha_problem, phi_q=None, phi_k=None) -> int:
    _, pq = _fm_ptr(phi_q)
    _, pk = _fm_ptr(phi_k)
    return _lib().hybrid_attn_validate(ctypes.byref(problem) if problem is not None else None, pq, pk)


def hybrid_attn_workspace_bytes(problem: ha_problem, phi_q=None, phi_k=None) -> int:
    _, pq = _fm_ptr(phi_q)
    _, pk = _fm_ptr(phi_k)
    return _lib().hybrid_attn_workspace_bytes(ctypes.byref(problem), pq, pk)


def hybrid_attn_value_distill_grad_workspace_bytes(problem: ha_problem, phi_q=None, phi_k=None) -> int:
    sq, pq = _fm_ptr(phi_q)
    sk, pk = _fm_ptr(phi_k)
    return _lib().hybrid_attn_value_distill_grad_workspace_bytes(ctypes.byref(problem), pq, pk)


def hybrid_attn_status_string(status: int) -> str:
    return _lib().hybrid_attn_status_string(status).decode()


def hybrid_attn_last_device_error() -> int:
    return _lib().hybrid_attn_last_device_error()


def hybrid_attn_abi_version() -> int:
    return _lib().hybrid_attn_abi_version()


def hybrid_attn_profile_enable(n_records: int) -> None:
    st = _lib().hybrid_attn_profile_enable(n_records)
    if st != HA_OK:
        raise HybridAttnError(st, "hybrid_attn_profile_enable")


def hybrid_attn_profile_count() -> int:
    return _lib().hybrid_attn_profile_count()



def hybrid_attn_mfma_probe(random_operands: bool, iters: int, launches: int, sink: torch.Tensor) -> float:
    """Enqueue the matrix-core probe on the current stream (see the header); returns the flops of one
    launch.  `sink`: device tensor of at least 2 KiB per compute unit."""
    flops = ctypes.c_double(0.0)
    st = _lib().hybrid_attn_mfma_probe(int(bool(random_operands)), iters, launches, sink.data_ptr(),
                                       sink.numel() * sink.element_size(), ctypes.byref(flops),
                                       torch.cuda.current_stream(sink.device).cuda_stream)
    if st != HA_OK:
        raise HybridAttnError(st, "hybrid_attn_mfma_probe")
    return flops.value



def hybrid_attn_select_rates(cost, error, budget: float):
    """Block-rate selection (Sec. 3.3): cost[i][r], error[i][r] per block i and candidate r (host
    numbers); returns (choice per block, total cost, total error) of the minimum-error assignment
    within the budget, or None when nothing fits."""
    n_blocks, n_rates = len(cost), len(cost[0])
    if any(len(c) != n_rates for c in cost) or len(error) != n_blocks or any(len(e) != n_rates for e in error):
        raise ValueError("cost and error must be n_blocks x n_rates tables of one shape")
    arr = ctypes.c_double * (n_blocks * n_rates)
    c = arr(*[float(x) for row in cost for x in row])
    e = arr(*[float(x) for row in error for x in row])
    choice = (ctypes.c_int * n_blocks)()
    tc, te = ctypes.c_double(0.0), ctypes.c_double(0.0)
    st = _lib().hybrid_attn_select_rates(n_blocks, n_rates, c, e, float(budget), choice, ctypes.byref(tc), ctypes.byref(te))
    if st == HA_ERR_INFEASIBLE:
        return None
    if st != HA_OK:
        raise HybridAttnError(st, "hybrid_attn_select_rates")
    return tuple(choice), tc.value, te.value


def hybrid_attn_profile_read(index: int):
    """Stage durations (ms) of recorded forward `index`: compaction, state, q-weight prep, query
    kernel, whole forward."""
    ms = (ctypes.c_float * 5)()
    st = _lib().hybrid_attn_profile_read(index, ms)
    if st != HA_OK:
        raise HybridAttnError(st, "hybrid_attn_profile_read")
    return list(ms)


def _require_gpu(*tensors):
    for t in tensors:
        if t is not None and not t.is_cuda:
            raise RuntimeError("hybrid_attn runs on the GPU only: got a CPU tensor (there is no CPU fallback)")


def _same_layout(q, *others):
    for t in others:
        if t.shape != q.shape or t.stride() != q.stride() or t.dtype != q.dtype:
            raise ValueError("q, k, v and out must share shape, strides and dtype")


def hybrid_attn_forward(q, k, v, phi_q: Optional[FeatureMap], phi_k: Optional[FeatureMap], hybrid_rate: int,
                        block_size: int = 128, softmax_scale: Optional[float] = None, out=None, workspace=None,
                        stream=None):
    """Enqueue one forward of Eq. "hybrid" (Sec. 3.2) on the current (or given) stream and return
    `out` ([B, H, N, d] with q's strides and dtype).  Does not synchronise."""
    _require_gpu(q, k, v)
    if softmax_scale is None:
        softmax_scale = float(q.shape[-1]) ** -0.5
    if out is None:
        with _alloc_on(stream):
            out = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device)
    _same_layout(q, k, v, out)
    prob = make_problem(q, hybrid_rate, block_size, softmax_scale)
    sq, pq = _fm_ptr(phi_q, q)
    sk, pk = _fm_ptr(phi_k, q)
    lib = _lib()
    st = lib.hybrid_attn_validate(ctypes.byref(prob), pq, pk)
    if st != HA_OK:
        raise HybridAttnError(st, "hybrid_attn_validate")
    need = lib.hybrid_attn_workspace_bytes(ctypes.byref(prob), pq, pk)
    if workspace is None:
        with _alloc_on(stream):
            workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    stream_handle = (stream if stream is not None else torch.cuda.current_stream(q.device)).cuda_stream
    st = lib.hybrid_attn_forward(ctypes.byref(prob), q.data_ptr(), k.data_ptr(), v.data_ptr(), pq, pk,
                                 out.data_ptr(), workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                 stream_handle)
    if st != HA_OK:
        raise HybridAttnError(st, "hybrid_attn_forward")
    return out



def hybrid_attn_static_scratch_bytes() -> int:
    return _lib().hybrid_attn_static_scratch_bytes()


def hybrid_attn_forward_static(q, k, v, phi_q: Optional[FeatureMap], phi_k: Optional[FeatureMap], hybrid_rate: int,
                               out, block_size: int = 128, softmax_scale: Optional[float] = None, stream=None):
    """hybrid_attn_forward for callers that cannot allocate: the library's static device array is the workspace and
    `out` is the caller's.  Nothing is allocated here or in the library.  Does not synchronise."""
    _require_gpu(q, k, v, out)
    if softmax_scale is None:
        softmax_scale = float(q.shape[-1]) ** -0.5
    _same_layout(q, k, v, out)
    prob = make_problem(q, hybrid_rate, block_size, softmax_scale)
    sq, pq = _fm_ptr(phi_q, q)
    sk, pk = _fm_ptr(phi_k, q)
    stream_handle = (stream if stream is not None else torch.cuda.current_stream(q.device)).cuda_stream
    st = _lib().hybrid_attn_forward_static(ctypes.byref(prob), q.data_ptr(), k.data_ptr(), v.data_ptr(), pq, pk,
                                           out.data_ptr(), stream_handle)
    if st != HA_OK:
        raise HybridAttnError(st, "hybrid_attn_forward_static")
    return out


@_allocations_follow_stream
def hybrid_attn_value_distill_loss(q, k, v, phi_q: Optional[FeatureMap], phi_k: Optional[FeatureMap], hybrid_rate: int,
                                   block_size: int = 128, softmax_scale: Optional[float] = None, y_teacher=None,
                                   teacher_is_cached: bool = False, y_student=None, workspace=None, stream=None):
    """Value-distillation loss of Sec. 3.3 (Eq. "vd_loss"): enqueues teacher forward (unless cached),
    student forward and the reduction; returns (loss, y_teacher, y_student) with `loss` a device
    float64 tensor [1 + B * H] (total, then per (batch, head)).  Does not synchronise."""
    _require_gpu(q, k, v)
    if softmax_scale is None:
        softmax_scale = float(q.shape[-1]) ** -0.5
    if y_teacher is None:
        if teacher_is_cached:
            raise ValueError("teacher_is_cached needs y_teacher")
        y_teacher = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device)
    if y_student is None:
        y_student = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device)
    _same_layout(q, k, v, y_teacher, y_student)
    prob = make_problem(q, hybrid_rate, block_size, softmax_scale)
    sq, pq = _fm_ptr(phi_q, q)
    sk, pk = _fm_ptr(phi_k, q)
    lib = _lib()
    st = lib.hybrid_attn_validate(ctypes.byref(prob), pq, pk)
    if st != HA_OK:
        raise HybridAttnError(st, "hybrid_attn_validate")
    need = lib.hybrid_attn_value_distill_workspace_bytes(ctypes.byref(prob), pq, pk)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    loss = torch.empty(1 + q.shape[0] * q.shape[1], dtype=torch.float64, device=q.device)
    stream_handle = (stream if stream is not None else torch.cuda.current_stream(q.device)).cuda_stream
    st = lib.hybrid_attn_value_distill_loss(ctypes.byref(prob), q.data_ptr(), k.data_ptr(), v.data_ptr(), pq, pk,
                                            int(teacher_is_cached), y_teacher.data_ptr(), y_student.data_ptr(),
                                            loss.data_ptr(), workspace.data_ptr(),
                                            workspace.numel() * workspace.element_size(), stream_handle)
    if st != HA_OK:
        raise HybridAttnError(st, "hybrid_attn_value_distill_loss")
    return loss, y_teacher, y_student


@_allocations_follow_stream
def hybrid_attn_value_distill_grad(q, k, v, phi_q: FeatureMap, phi_k: FeatureMap, hybrid_rate: int, block_size: int = 128,
                                   softmax_scale: Optional[float] = None, y_teacher=None, teacher_is_cached: bool = False,
                                   y_student=None, row_den=None, student_is_cached: bool = False, workspace=None,
                                   stream=None):
    """Loss and gradient of the value-distillation step (Sec. 3.3, Alg. 1): returns (loss, grads_q, grads_k, y_teacher,
    y_student, row_den); grads_* is a dict of fp32 device tensors w1 [H, Hd, d], b1 [H, Hd], w2 [H, F, Hd], b2 [H, F]
    summed over the batch.  Does not synchronise."""
    _require_gpu(q, k, v)
    if softmax_scale is None:
        softmax_scale = float(q.shape[-1]) ** -0.5
    if y_teacher is None:
        if teacher_is_cached:
            raise ValueError("teacher_is_cached needs y_teacher")
        y_teacher = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device)
    if student_is_cached and (y_student is None or row_den is None):
        raise ValueError("student_is_cached needs y_student and row_den")
    if y_student is None:
        y_student = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device)
    if row_den is None:
        row_den = torch.empty(q.shape[:3], dtype=torch.float32, device=q.device)
    if row_den.dtype != torch.float32 or not row_den.is_contiguous() or tuple(row_den.shape) != tuple(q.shape[:3]):
        raise ValueError("row_den must be a contiguous fp32 tensor [B, H, N]")
    _same_layout(q, k, v, y_teacher, y_student)
    prob = make_problem(q, hybrid_rate, block_size, softmax_scale)
    sq, pq = _fm_ptr(phi_q, q)
    sk, pk = _fm_ptr(phi_k, q)
    lib = _lib()
    need = lib.hybrid_attn_value_distill_grad_workspace_bytes(ctypes.byref(prob), pq, pk)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    B, H = q.shape[0], q.shape[1]
    loss = torch.empty(1 + B * H, dtype=torch.float64, device=q.device)

    def grads_of(fm):
        t = dict(w1=torch.empty(fm.w1.shape, dtype=torch.float32, device=q.device),
                 b1=torch.empty(fm.w1.shape[:2], dtype=torch.float32, device=q.device),
                 w2=torch.empty(fm.w2.shape, dtype=torch.float32, device=q.device),
                 b2=torch.empty(fm.w2.shape[:2], dtype=torch.float32, device=q.device))
        if fm.w_mid is not None:
            t["w_mid"] = torch.empty(fm.w_mid.shape, dtype=torch.float32, device=q.device)
            t["b_mid"] = torch.empty(fm.w_mid.shape[:2], dtype=torch.float32, device=q.device)
        return t, ha_feature_map_grad(t["w1"].data_ptr(), t["b1"].data_ptr(), t["w2"].data_ptr(), t["b2"].data_ptr(),
                                      t["w_mid"].data_ptr() if "w_mid" in t else None,
                                      t["b_mid"].data_ptr() if "b_mid" in t else None)

    gq, cq = grads_of(phi_q)
    gk, ck = grads_of(phi_k)
    stream_handle = (stream if stream is not None else torch.cuda.current_stream(q.device)).cuda_stream
    st = lib.hybrid_attn_value_distill_grad(ctypes.byref(prob), q.data_ptr(), k.data_ptr(), v.data_ptr(), pq, pk,
                                            int(teacher_is_cached), int(student_is_cached), y_teacher.data_ptr(),
                                            y_student.data_ptr(), row_den.data_ptr(), loss.data_ptr(), ctypes.byref(cq),
                                            ctypes.byref(ck), workspace.data_ptr(),
                                            workspace.numel() * workspace.element_size(), stream_handle)
    if st != HA_OK:
        raise HybridAttnError(st, "hybrid_attn_value_distill_grad")
    return loss, gq, gk, y_teacher, y_student, row_den


def hybrid_attn_param_update(master, grad, lr: float, kind: int = HA_OPT_SGD, m=None, v=None, step: int = 1,
                             grad_scale: float = 1.0, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8,
                             weight_decay: float = 0.01, param_io=None, stream=None):
    """One update (Alg. 1's phi <- phi - eta grad, or AdamW) of one parameter tensor, in place: master (fp32), the
    moments m, v (AdamW) and, if given, param_io (bf16 or fp32 tensor of the same shape that the forward reads)."""
    _require_gpu(master, grad)
    for t in (master, grad, m, v):
        if t is not None and (t.dtype != torch.float32 or not t.is_contiguous() or t.numel() != master.numel()):
            raise ValueError("master, grad, m, v must be contiguous fp32 tensors of one size")
    io_code = HA_BF16
    if param_io is not None:
        if not param_io.is_contiguous() or param_io.numel() != master.numel():
            raise ValueError("param_io must be contiguous and of master's size")
        io_code = _dtype_code(param_io)
    opt = ha_optimizer(kind, step, lr, grad_scale, beta1, beta2, eps, weight_decay)
    stream_handle = (stream if stream is not None else torch.cuda.current_stream(master.device)).cuda_stream
    st = _lib().hybrid_attn_param_update(ctypes.byref(opt), master.numel(), master.data_ptr(), grad.data_ptr(),
                                         m.data_ptr() if m is not None else None, v.data_ptr() if v is not None else None,
                                         param_io.data_ptr() if param_io is not None else None, io_code, stream_handle)
    if st != HA_OK:
        raise HybridAttnError(st, "hybrid_attn_param_update")


@_allocations_follow_stream
def hybrid_attn_linear_state(k, v, phi_k: FeatureMap, hybrid_rate: int, block_size: int = 128, workspace=None,
                             stream=None):
    """Key-side passes only: returns (S [B, H, F, d], z [B, H, F]) in fp32 (test tap)."""
    _require_gpu(k, v)
    _same_layout(k, v)
    prob = make_problem(k, hybrid_rate, block_size, 1.0)
    sk, pk = _fm_ptr(phi_k, k)
    lib = _lib()
    need = lib.hybrid_attn_workspace_bytes(ctypes.byref(prob), pk, pk)
    if need == 0:
        raise HybridAttnError(lib.hybrid_attn_validate(ctypes.byref(prob), pk, pk), "hybrid_attn_validate")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=k.device)
    B, H, N, d = k.shape
    S = torch.empty(B, H, sk.d_out, d, dtype=torch.float32, device=k.device)
    z = torch.empty(B, H, sk.d_out, dtype=torch.float32, device=k.device)
    stream_handle = (stream if stream is not None else torch.cuda.current_stream(k.device)).cuda_stream
    st = lib.hybrid_attn_linear_state(ctypes.byref(prob), k.data_ptr(), v.data_ptr(), pk, S.data_ptr(), z.data_ptr(),
                                      workspace.data_ptr(), workspace.numel(), stream_handle)
    if st != HA_OK:
        raise HybridAttnError(st, "hybrid_attn_linear_state")
    return S, z


def to_device(inputs, device="cuda"):
    """workloads.Inputs (numpy float32) -> device tensors in the workload's io dtype."""
    w = inputs.workload
    dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32

    def dev(a, dtype):
        return torch.from_numpy(a).to(device=device, dtype=dtype).contiguous()

    def fm(p):
        mid = getattr(p, "w_mid", None)
        return FeatureMap(dev(p.w1, dt), dev(p.b1, torch.float32), dev(p.w2, dt), dev(p.b2, torch.float32),
                          p.poly_degree, w_mid=dev(mid, dt) if mid is not None else None,
                          b_mid=dev(p.b_mid, torch.float32) if mid is not None else None)
    return dev(inputs.q, dt), dev(inputs.k, dt), dev(inputs.v, dt), fm(inputs.phi_q), fm(inputs.phi_k)


def device_inputs(w, device="cuda"):
    """workloads.make_inputs_on_device as (q, k, v, FeatureMap phi_q, FeatureMap phi_k)."""
    from . import workloads as W
    q, k, v, mq, mk = W.make_inputs_on_device(w, device)

    def fm(m):
        return FeatureMap(m["w1"], m["b1"], m["w2"], m["b2"], w.poly_degree, w_mid=m.get("w_mid"), b_mid=m.get("b_mid"))
    return q, k, v, fm(mq), fm(mk)
