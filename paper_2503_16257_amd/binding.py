"""ctypes binding of libvidkv.so: same names as the C ABI, argument marshalling only.

Every step of the path runs in the library's HIP kernels; this module checks
tensor dtype / device / contiguity, takes data pointers and the current
stream, and turns a non-zero status into an exception.  If the library has not
been built the first call raises: there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import math
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libvidkv.so")

OK, EINVAL, ESHAPE, ENOSPACE, EHIP = 0, 1, 2, 3, 4


ABI_VERSION = 3          # VIDKV_ABI_VERSION of include/vidkv.h that this binding was written for


class VidkvParams(C.Structure):
    _fields_ = [
        ("n_layers", C.c_int32), ("batch", C.c_int32), ("n_kv_heads", C.c_int32),
        ("n_q_heads", C.c_int32), ("head_dim", C.c_int32), ("group", C.c_int32),
        ("t_quant", C.c_int32), ("n_anom", C.c_int32), ("use_fft", C.c_int32),
        ("n_salient", C.c_int32), ("gamma", C.c_float), ("softmax_scale", C.c_float),
        ("t_capacity", C.c_int32), ("salient_bits", C.c_int32), ("channel_metric", C.c_int32),
    ]


class VidkvSideStream(C.Structure):
    _fields_ = [("hip_stream", C.c_void_p), ("fork_event", C.c_void_p), ("join_event", C.c_void_p)]


class SideStream:
    """A torch stream and two events for the calls that take a vidkv_side_stream.

    Owned by the caller: keep it alive as long as work enqueued with it may run."""

    def __init__(self, device="cuda:0"):
        import torch
        with torch.cuda.device(device):
            self.stream = torch.cuda.Stream(device=device)          # default priority
            self.fork = torch.cuda.Event(enable_timing=False)
            self.join = torch.cuda.Event(enable_timing=False)
            # torch creates the event handle lazily, at the first record
            self.fork.record(self.stream)
            self.join.record(self.stream)
        self.c = VidkvSideStream(self.stream.cuda_stream, self.fork.cuda_event, self.join.cuda_event)


def _side(side):
    return None if side is None else C.byref(side.c)


class VidkvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


_lib = None


def lib() -> C.CDLL:
    """Load the shared library (once).  Raises if it is not built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2503_16257_amd.build`")
        # PyTorch ships its own HIP runtime; it must be in the process before this library is
        # loaded, so that both resolve to that one copy.  Loaded the other way round the
        # library registers its kernels with a second runtime, and every launch on a torch
        # stream fails.
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        PP = C.POINTER(VidkvParams)
        vp, sz, i32 = C.c_void_p, C.c_size_t, C.c_int32
        L.vidkv_packed_keys_bytes.argtypes = [PP]
        L.vidkv_packed_keys_bytes.restype = sz
        L.vidkv_packed_values_bytes.argtypes = [PP]
        L.vidkv_packed_values_bytes.restype = sz
        L.vidkv_workspace_bytes.argtypes = [PP, C.c_int]
        L.vidkv_workspace_bytes.restype = sz
        L.vidkv_quantize_keys.argtypes = [PP, vp, vp, sz, vp, sz, vp]
        L.vidkv_quantize_keys.restype = C.c_int
        L.vidkv_quantize_values.argtypes = [PP, vp, vp, vp, vp, sz, vp, sz, vp]
        L.vidkv_quantize_values.restype = C.c_int
        SP = C.POINTER(VidkvSideStream)
        L.vidkv_quantize_kv.argtypes = [PP, vp, vp, vp, vp, vp, sz, vp, sz, vp, sz, vp, SP]
        L.vidkv_quantize_kv.restype = C.c_int
        L.vidkv_flush_residual.argtypes = [PP, i32, vp, vp, i32, i32, vp, sz, vp, sz, vp]
        L.vidkv_flush_residual.restype = C.c_int
        L.vidkv_saliency_workspace_bytes.argtypes = [i32, i32]
        L.vidkv_saliency_workspace_bytes.restype = sz
        L.vidkv_saliency_scores.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, sz, vp]
        L.vidkv_saliency_scores.restype = C.c_int
        L.vidkv_decode_attention.argtypes = [PP, i32, vp, vp, vp, vp, vp, i32, vp, vp, vp, sz, vp, SP]
        L.vidkv_decode_attention.restype = C.c_int
        L.vidkv_decode_attention_noalloc.argtypes = [PP, i32, vp, vp, vp, vp, vp, i32, vp, vp, vp]
        L.vidkv_decode_attention_noalloc.restype = C.c_int
        u32 = C.c_uint32
        L.vidkv_quantize_keys_stages.argtypes = [PP, vp, vp, sz, vp, sz, u32, vp]
        L.vidkv_quantize_keys_stages.restype = C.c_int
        L.vidkv_quantize_values_stages.argtypes = [PP, vp, vp, vp, vp, sz, vp, sz, u32, vp]
        L.vidkv_quantize_values_stages.restype = C.c_int
        L.vidkv_decode_attention_stages.argtypes = [PP, i32, vp, vp, vp, vp, vp, i32, vp, vp, vp,
                                                    sz, u32, vp, SP]
        L.vidkv_decode_attention_stages.restype = C.c_int
        L.vidkv_calib_copy.argtypes = [vp, vp, sz, vp]
        L.vidkv_calib_copy.restype = C.c_int
        L.vidkv_status_string.argtypes = [C.c_int]
        L.vidkv_status_string.restype = C.c_char_p
        L.vidkv_abi_version.argtypes = []
        L.vidkv_abi_version.restype = C.c_int
        _lib = L
    return _lib


def make_params(n_layers, batch, n_kv_heads, n_q_heads, t_quant, n_anom, n_salient,
                gamma=0.7, softmax_scale=None, head_dim=128, group=32, use_fft=1,
                t_capacity=0, salient_bits=0, channel_metric=0) -> VidkvParams:
    if softmax_scale is None:
        softmax_scale = 1.0 / math.sqrt(head_dim)
    return VidkvParams(n_layers, batch, n_kv_heads, n_q_heads, head_dim, group, t_quant, n_anom,
                       use_fft, n_salient, gamma, softmax_scale, t_capacity, salient_bits, channel_metric)


def status_string(status: int) -> str:
    return lib().vidkv_status_string(status).decode()


def abi_version() -> int:
    return lib().vidkv_abi_version()


def packed_keys_bytes(p: VidkvParams) -> int:
    return lib().vidkv_packed_keys_bytes(C.byref(p))


def packed_values_bytes(p: VidkvParams) -> int:
    return lib().vidkv_packed_values_bytes(C.byref(p))


def workspace_bytes(p: VidkvParams, which: int) -> int:
    return lib().vidkv_workspace_bytes(C.byref(p), which)


def _ptr(t, dtype=None, name="tensor"):
    """Device pointer of a contiguous CUDA tensor (None -> NULL)."""
    if t is None:
        return None
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name}: expected a CUDA tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name}: must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name}: expected dtype {dtype}, got {t.dtype}")
    return C.c_void_p(t.data_ptr())


def _nbytes(t) -> int:
    return t.numel() * t.element_size()


def _stream(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _check(status: int, where: str):
    if status != OK:
        raise VidkvError(status, where)


def quantize_keys(p: VidkvParams, K, packed_K, workspace, stream=None, stages=None) -> None:
    """vidkv_quantize_keys: K [L,B,Hkv,Tq,128] fp16 -> packed_K (uint8 buffer).
    With `stages` (bit mask) calls vidkv_quantize_keys_stages instead."""
    import torch
    a = [C.byref(p), _ptr(K, torch.float16, "K"), _ptr(packed_K, torch.uint8, "packed_K"),
         _nbytes(packed_K), _ptr(workspace, torch.uint8, "workspace"), _nbytes(workspace)]
    if stages is None:
        _check(lib().vidkv_quantize_keys(*a, _stream(stream)), "vidkv_quantize_keys")
    else:
        _check(lib().vidkv_quantize_keys_stages(*a, stages, _stream(stream)),
               "vidkv_quantize_keys_stages")


def quantize_values(p: VidkvParams, V, packed_V, workspace, saliency=None, salient_idx=None,
                    stream=None, stages=None) -> None:
    """vidkv_quantize_values: V fp16 (+ scores [B,Tq] f32 or indices [B,n_s] i32) -> packed_V."""
    import torch
    a = [C.byref(p), _ptr(V, torch.float16, "V"), _ptr(saliency, torch.float32, "saliency"),
         _ptr(salient_idx, torch.int32, "salient_idx"), _ptr(packed_V, torch.uint8, "packed_V"),
         _nbytes(packed_V), _ptr(workspace, torch.uint8, "workspace"), _nbytes(workspace)]
    if stages is None:
        _check(lib().vidkv_quantize_values(*a, _stream(stream)), "vidkv_quantize_values")
    else:
        _check(lib().vidkv_quantize_values_stages(*a, stages, _stream(stream)),
               "vidkv_quantize_values_stages")


def decode_attention(p: VidkvParams, layer: int, q, packed_K, packed_V, out, workspace,
                     K_tail=None, V_tail=None, tail_capacity: int = 0, tail_len=None,
                     stream=None, stages=None, side=None) -> None:
    """vidkv_decode_attention: one decode step of one layer -> out [B,Hq,128] fp16.
    `side`: a SideStream for the residual-token kernel of a large block, or None (in line)."""
    import torch
    a = [C.byref(p), layer, _ptr(q, torch.float16, "q"), _ptr(packed_K, torch.uint8, "packed_K"),
         _ptr(packed_V, torch.uint8, "packed_V"), _ptr(K_tail, torch.float16, "K_tail"),
         _ptr(V_tail, torch.float16, "V_tail"), tail_capacity, _ptr(tail_len, torch.int32, "tail_len"),
         _ptr(out, torch.float16, "out"), _ptr(workspace, torch.uint8, "workspace"),
         _nbytes(workspace)]
    if stages is None:
        _check(lib().vidkv_decode_attention(*a, _stream(stream), _side(side)), "vidkv_decode_attention")
    else:
        _check(lib().vidkv_decode_attention_stages(*a, stages, _stream(stream), _side(side)),
               "vidkv_decode_attention_stages")


NOALLOC_SCRATCH_BYTES = 16 << 20     # VIDKV_NOALLOC_SCRATCH_BYTES of include/vidkv.h


def decode_attention_noalloc(p: VidkvParams, layer: int, q, packed_K, packed_V, out, K_tail=None,
                             V_tail=None, tail_capacity: int = 0, tail_len=None, stream=None) -> None:
    """vidkv_decode_attention_noalloc: the decode step without a workspace argument."""
    import torch
    _check(lib().vidkv_decode_attention_noalloc(
        C.byref(p), layer, _ptr(q, torch.float16, "q"), _ptr(packed_K, torch.uint8, "packed_K"),
        _ptr(packed_V, torch.uint8, "packed_V"), _ptr(K_tail, torch.float16, "K_tail"),
        _ptr(V_tail, torch.float16, "V_tail"), tail_capacity, _ptr(tail_len, torch.int32, "tail_len"),
        _ptr(out, torch.float16, "out"), _stream(stream)), "vidkv_decode_attention_noalloc")


def quantize_kv(p: VidkvParams, K, V, packed_K, packed_V, workspace, saliency=None,
                salient_idx=None, stream=None, side=None) -> None:
    """vidkv_quantize_kv: both tensors of the same tokens in one call.
    `side`: a SideStream for the protected-token selection, or None (in line)."""
    import torch
    _check(lib().vidkv_quantize_kv(
        C.byref(p), _ptr(K, torch.float16, "K"), _ptr(V, torch.float16, "V"),
        _ptr(saliency, torch.float32, "saliency"), _ptr(salient_idx, torch.int32, "salient_idx"),
        _ptr(packed_K, torch.uint8, "packed_K"), _nbytes(packed_K),
        _ptr(packed_V, torch.uint8, "packed_V"), _nbytes(packed_V),
        _ptr(workspace, torch.uint8, "workspace"), _nbytes(workspace), _stream(stream), _side(side)),
        "vidkv_quantize_kv")


def flush_residual(p: VidkvParams, layer: int, K_tail, V_tail, tail_capacity: int, n_flush: int,
                   packed_K, packed_V, stream=None) -> None:
    """vidkv_flush_residual: code the first n_flush residual tokens of one layer and append them."""
    import torch
    _check(lib().vidkv_flush_residual(
        C.byref(p), layer, _ptr(K_tail, torch.float16, "K_tail"), _ptr(V_tail, torch.float16, "V_tail"),
        tail_capacity, n_flush, _ptr(packed_K, torch.uint8, "packed_K"), _nbytes(packed_K),
        _ptr(packed_V, torch.uint8, "packed_V"), _nbytes(packed_V), _stream(stream)),
        "vidkv_flush_residual")


def saliency_workspace_bytes(batch: int, hidden_dim: int) -> int:
    return lib().vidkv_saliency_workspace_bytes(batch, hidden_dim)


def saliency_scores(X_v, X_t, scores, workspace, stream=None) -> None:
    """vidkv_saliency_scores: X_v [B,Tv,d] fp16, X_t [B,Nt,d] fp16 -> scores [B,Tv] f32."""
    import torch
    B, Tv, d = X_v.shape
    assert X_t.shape[0] == B and X_t.shape[2] == d and tuple(scores.shape) == (B, Tv)
    _check(lib().vidkv_saliency_scores(
        _ptr(X_v, torch.float16, "X_v"), _ptr(X_t, torch.float16, "X_t"), B, Tv, X_t.shape[1], d,
        _ptr(scores, torch.float32, "scores"), _ptr(workspace, torch.uint8, "workspace"),
        _nbytes(workspace), _stream(stream)), "vidkv_saliency_scores")


def calib_copy(dst, src, stream=None) -> None:
    _check(lib().vidkv_calib_copy(_ptr(dst, None, "dst"), _ptr(src, None, "src"), _nbytes(src),
                                  _stream(stream)), "vidkv_calib_copy")


def alloc_bytes(nbytes: int, device="cuda:0"):
    """A 256-byte-aligned uint8 device buffer (torch's allocator aligns to 512)."""
    import torch
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)
