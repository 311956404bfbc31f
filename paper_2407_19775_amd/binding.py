"""ctypes binding of libmmd8.so: argument marshalling only.

Every function takes torch tensors that already live on the GPU, passes their addresses,
shapes and strides through the C ABI (include/mmd8.h) on torch's current HIP stream, and
raises on a non-zero status.  There is no CPU fallback: if the library has not been built the
first call raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmmd8.so")
_lib = None

EXPORTS = (
    "mmd8_status_string", "mmd8_quantize_blockwise", "mmd8_dequantize_blockwise", "mmd8_code_table",
    "mmd8_code_midpoints", "mmd8_packed_weight_layout", "mmd8_packed_weight_bytes", "mmd8_prequantize_weight",
    "mmd8_unpack_weight", "mmd8_linear_workspace_bytes", "mmd8_linear_workspace_init", "mmd8_mixed_int8_linear",
    "mmd8_threshold_fp16_pattern", "mmd8_mixed_int8_linear_from_codes", "mmd8_linear_lora_workspace_bytes",
    "mmd8_mixed_int8_linear_lora", "mmd8_linear_to_codes_workspace_bytes", "mmd8_mixed_int8_linear_to_codes",
    "mmd8_mixed_int8_linear_gelu", "mmd8_mixed_int8_linear_residual", "mmd8_mixed_int8_linear_static",
    "mmd8_mixed_int8_linear_readings", "mmd8_quantize_blockwise_h", "mmd8_dequantize_blockwise_h",
)


class DebugTaps(ctypes.Structure):
    _fields_ = [(name, ctypes.c_void_p) for name in
                ("outlier_mask", "row_absmax", "xq", "acc", "n_outliers", "outlier_idx",
                 "event_begin", "event_prep_mid", "event_gemm_begin", "event_gemm_end")] + [("tuning", ctypes.c_uint32)]


class Readings(ctypes.Structure):
    _fields_ = [("row_scale", ctypes.c_int), ("W_master", ctypes.c_void_p), ("ldw", ctypes.c_int)]


ROW_SCALE_SUB_THRESHOLD, ROW_SCALE_NON_CRITICAL = 0, 1

# kernel choices of one call (mmd8_debug_taps.tuning, include/mmd8.h)
TUNE_SEPARATE_PREP = 0x10
TUNE_NO_ROWS_KERNEL = 0x20


def tune_gemm_tiles(v: int) -> int:
    return (v + 1) & 0xF


class Mmd8Error(RuntimeError):
    pass


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise Mmd8Error("libmmd8.so is not built: run `python -m paper_2407_19775_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, sz, i32, f32, u32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_float, ctypes.c_uint32
        L.mmd8_status_string.restype = ctypes.c_char_p
        L.mmd8_status_string.argtypes = [i32]
        L.mmd8_quantize_blockwise.argtypes = [vp, sz, i32, vp, vp, vp]
        L.mmd8_dequantize_blockwise.argtypes = [vp, vp, sz, i32, vp, vp]
        L.mmd8_quantize_blockwise_h.argtypes = [vp, sz, i32, vp, vp, vp]
        L.mmd8_dequantize_blockwise_h.argtypes = [vp, vp, sz, i32, vp, vp]
        L.mmd8_code_table.restype = ctypes.POINTER(ctypes.c_float)
        L.mmd8_code_midpoints.restype = ctypes.POINTER(ctypes.c_float)
        L.mmd8_packed_weight_layout.restype = ctypes.c_uint32
        L.mmd8_packed_weight_bytes.restype = sz
        L.mmd8_packed_weight_bytes.argtypes = [i32, i32]
        L.mmd8_prequantize_weight.argtypes = [vp, i32, i32, i32, vp, vp, vp]
        L.mmd8_unpack_weight.argtypes = [vp, u32, i32, i32, vp, vp]
        L.mmd8_linear_workspace_bytes.restype = sz
        L.mmd8_linear_workspace_bytes.argtypes = [i32, i32, i32]
        L.mmd8_linear_workspace_init.argtypes = [vp, sz, vp]
        L.mmd8_mixed_int8_linear.argtypes = [vp, i32, i32, i32, vp, u32, vp, i32, vp, f32, vp, i32, vp, sz,
                                             ctypes.POINTER(DebugTaps), vp]
        L.mmd8_mixed_int8_linear_static.argtypes = [vp, i32, i32, i32, vp, u32, vp, i32, vp, f32, vp, i32,
                                                    ctypes.POINTER(DebugTaps), vp]
        L.mmd8_mixed_int8_linear_readings.argtypes = [vp, i32, i32, i32, vp, u32, vp, i32, vp, f32, ctypes.POINTER(Readings),
                                                      vp, i32, vp, sz, ctypes.POINTER(DebugTaps), vp]
        L.mmd8_mixed_int8_linear_from_codes.argtypes = [vp, vp, i32, i32, i32, vp, vp, u32, vp, i32, vp, f32, vp, i32, vp, sz,
                                                        ctypes.POINTER(DebugTaps), vp]
        L.mmd8_linear_lora_workspace_bytes.restype = sz
        L.mmd8_linear_lora_workspace_bytes.argtypes = [i32, i32, i32, i32]
        L.mmd8_mixed_int8_linear_lora.argtypes = [vp, i32, i32, i32, vp, u32, vp, i32, vp, f32, vp, vp, i32, vp, vp, i32, vp, sz,
                                                  ctypes.POINTER(DebugTaps), vp]
        L.mmd8_mixed_int8_linear_gelu.argtypes = L.mmd8_mixed_int8_linear.argtypes
        L.mmd8_mixed_int8_linear_residual.argtypes = [vp, i32, i32, i32, vp, u32, vp, i32, vp, f32, vp, i32, vp, i32, vp, sz,
                                                      ctypes.POINTER(DebugTaps), vp]
        L.mmd8_linear_to_codes_workspace_bytes.restype = sz
        L.mmd8_linear_to_codes_workspace_bytes.argtypes = [i32, i32, i32, i32]
        L.mmd8_mixed_int8_linear_to_codes.argtypes = [vp, i32, i32, i32, vp, u32, vp, i32, vp, f32, vp, i32, i32, vp, vp, vp, vp, sz,
                                                      ctypes.POINTER(DebugTaps), vp]
        L.mmd8_threshold_fp16_pattern.restype = ctypes.c_uint32
        L.mmd8_threshold_fp16_pattern.argtypes = [f32]
        _lib = L
    return _lib


def _check(status: int):
    if status != 0:
        raise Mmd8Error("mmd8 status %d: %s" % (status, lib().mmd8_status_string(status).decode()))


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t: torch.Tensor, dtype, name: str):
    if not (t.is_cuda and t.dtype == dtype):
        raise Mmd8Error("%s must be a GPU tensor of dtype %s" % (name, dtype))
    return t


def code_table() -> torch.Tensor:
    return torch.tensor([lib().mmd8_code_table()[i] for i in range(256)], dtype=torch.float32)


def code_midpoints() -> torch.Tensor:
    return torch.tensor([lib().mmd8_code_midpoints()[i] for i in range(255)], dtype=torch.float32)


# ------------------------------------------------------------------ blockwise codec
def quantize_blockwise(x: torch.Tensor, block: int, codes: torch.Tensor = None, absmax: torch.Tensor = None,
                       fp16_scales: bool = False):
    """x: fp16 GPU tensor (contiguous, any shape) -> (codes uint8 [n], absmax float32 [ceil(n/block)]).
    fp16_scales: the block scales as fp16 numbers (2 bytes per block) instead of fp32."""
    _dev(x, torch.float16, "x")
    if not x.is_contiguous():
        raise Mmd8Error("x must be contiguous")
    n = x.numel()
    nblk = (n + block - 1) // block if block > 0 else 0
    if codes is None:
        codes = torch.empty(n, dtype=torch.uint8, device=x.device)
    sdt = torch.float16 if fp16_scales else torch.float32
    if absmax is None:
        absmax = torch.empty(nblk, dtype=sdt, device=x.device)
    _dev(absmax, sdt, "absmax")
    fn = lib().mmd8_quantize_blockwise_h if fp16_scales else lib().mmd8_quantize_blockwise
    _check(fn(x.data_ptr(), n, block, codes.data_ptr(), absmax.data_ptr(), _stream()))
    return codes, absmax


def dequantize_blockwise(codes: torch.Tensor, absmax: torch.Tensor, block: int, out: torch.Tensor = None):
    _dev(codes, torch.uint8, "codes")
    if absmax.dtype == torch.float16:           # block scales stored as fp16 numbers
        fn = lib().mmd8_dequantize_blockwise_h
    else:
        _dev(absmax, torch.float32, "absmax")
        fn = lib().mmd8_dequantize_blockwise
    n = codes.numel()
    if out is None:
        out = torch.empty(n, dtype=torch.float16, device=codes.device)
    _check(fn(codes.data_ptr(), absmax.data_ptr(), n, block, out.data_ptr(), _stream()))
    return out


# ------------------------------------------------------------------ mixed int8 linear
class PackedWeight:
    """Pre-quantized weight: opaque int8 blob + per-column absmax + the layout tag the blob was written under
    (handed back to every call that reads the blob, which refuses a tag that is not the library's own)."""

    def __init__(self, blob, col_absmax, K, N, layout=None):
        self.blob, self.col_absmax, self.K, self.N = blob, col_absmax, K, N
        self.layout = lib().mmd8_packed_weight_layout() if layout is None else int(layout)


def prequantize_weight(W: torch.Tensor) -> PackedWeight:
    """W: fp16 GPU tensor [K, N] (row stride may exceed N)."""
    _dev(W, torch.float16, "W")
    K, N = W.shape
    if W.stride(1) != 1:
        raise Mmd8Error("W must have unit stride along N")
    nbytes = lib().mmd8_packed_weight_bytes(K, N)
    if nbytes == 0:
        _check(-2)
    blob = torch.empty(nbytes, dtype=torch.int8, device=W.device)
    c = torch.empty(N, dtype=torch.float32, device=W.device)
    _check(lib().mmd8_prequantize_weight(W.data_ptr(), K, N, W.stride(0), blob.data_ptr(), c.data_ptr(), _stream()))
    return PackedWeight(blob, c, K, N)


def unpack_weight(pw: PackedWeight) -> torch.Tensor:
    out = torch.empty((pw.K, pw.N), dtype=torch.int8, device=pw.blob.device)
    _check(lib().mmd8_unpack_weight(pw.blob.data_ptr(), pw.layout, pw.K, pw.N, out.data_ptr(), _stream()))
    return out


def linear_workspace(M: int, K: int, N: int, device, lora_rank: int = 0, exit_block: int = 0) -> torch.Tensor:
    """Allocates and sets up a workspace large enough for one [M,K] x [K,N] call (with an adapter of
    rank lora_rank, if not 0; for an output leaving in coded form with blocks of exit_block, if not 0)."""
    if lora_rank and exit_block:
        raise Mmd8Error("an adapter and a coded output cannot be combined in one call")
    nbytes = (lib().mmd8_linear_lora_workspace_bytes(M, K, N, lora_rank) if lora_rank
              else lib().mmd8_linear_to_codes_workspace_bytes(M, K, N, exit_block) if exit_block
              else lib().mmd8_linear_workspace_bytes(M, K, N))
    if nbytes == 0:
        _check(-2)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
    _check(lib().mmd8_linear_workspace_init(ws.data_ptr(), ws.numel(), _stream()))
    return ws


def _taps(M, K, N, dev, only=None):
    """Buffers for the debug taps; only: names to keep (the others are not asked for)."""
    all_taps = _all_taps(M, K, N, dev)
    return all_taps if only is None else {k: all_taps[k] for k in only}


def _all_taps(M, K, N, dev):
    return dict(
        outlier_mask=torch.zeros(K, dtype=torch.uint8, device=dev),
        row_absmax=torch.zeros(M, dtype=torch.float32, device=dev),
        xq=torch.zeros((M, K), dtype=torch.int8, device=dev),
        acc=torch.zeros((M, N), dtype=torch.int32, device=dev),
        n_outliers=torch.zeros(1, dtype=torch.int32, device=dev),
        outlier_idx=torch.zeros(K, dtype=torch.int32, device=dev),
    )


def mixed_int8_linear_to_codes(X: torch.Tensor, pw: PackedWeight, tau: float, block: int, bias: torch.Tensor = None,
                               residual: torch.Tensor = None, codes: torch.Tensor = None, absmax: torch.Tensor = None,
                               H: torch.Tensor = None, workspace: torch.Tensor = None, taps: bool = False,
                               events=None, tuning: int = 0):
    """The layer with its result leaving blockwise-coded: H = Y (+ residual, an fp16 addition), flattened row by
    row and encoded with blocks of `block` elements.  Returns (codes [M N] uint8, absmax float32); H, if given
    (contiguous [M, N] fp16), receives the encoded tensor itself.  With taps=True the intermediates of the layer
    come back as a third value."""
    _dev(X, torch.float16, "X")
    M, K = X.shape
    if K != pw.K or X.stride(1) != 1:
        raise Mmd8Error("X must be [M, %d] with unit stride along K" % pw.K)
    N = pw.N
    n = M * N
    if codes is None:
        codes = torch.empty(n, dtype=torch.uint8, device=X.device)
    if absmax is None:
        absmax = torch.empty((n + block - 1) // max(block, 1), dtype=torch.float32, device=X.device)
    _dev(codes, torch.uint8, "codes")
    _dev(absmax, torch.float32, "absmax")
    if codes.numel() < n or absmax.numel() < (n + block - 1) // max(block, 1):
        raise Mmd8Error("codes / absmax too small")
    if residual is not None:
        _dev(residual, torch.float16, "residual")
        if residual.shape != (M, N) or residual.stride(1) != 1:
            raise Mmd8Error("residual must be [M, N] with unit stride along N")
    if H is not None and not (H.is_cuda and H.dtype == torch.float16 and H.shape == (M, N) and H.is_contiguous()):
        raise Mmd8Error("H must be a contiguous GPU fp16 tensor [M, N]")
    if workspace is None:
        workspace = linear_workspace(M, K, N, X.device, exit_block=block)
    tensors = _taps(M, K, N, X.device) if taps else None
    tp = DebugTaps(**{k: v.data_ptr() for k, v in tensors.items()}) if taps else None
    if events is not None and not taps:         # (begin, gemm_begin, gemm_end[, prep_mid]) hipEvent_t handles as ints
        tp = DebugTaps(event_begin=events[0], event_gemm_begin=events[1], event_gemm_end=events[2],
                       event_prep_mid=events[3] if len(events) > 3 else None)
    if tuning:
        tp = tp if tp is not None else DebugTaps()
        tp.tuning = int(tuning)
    _check(lib().mmd8_mixed_int8_linear_to_codes(
        X.data_ptr(), M, K, X.stride(0) if M > 0 else K, pw.blob.data_ptr(), pw.layout, pw.col_absmax.data_ptr(), N,
        bias.data_ptr() if bias is not None else None, float(tau),
        residual.data_ptr() if residual is not None else None,
        residual.stride(0) if residual is not None and M > 0 else N, int(block), codes.data_ptr(), absmax.data_ptr(),
        H.data_ptr() if H is not None else None, workspace.data_ptr(), workspace.numel(),
        ctypes.byref(tp) if tp is not None else None, _stream()))
    return (codes, absmax, tensors) if taps else (codes, absmax)


def mixed_int8_linear(X: torch.Tensor, pw: PackedWeight, tau: float, bias: torch.Tensor = None,
                      out: torch.Tensor = None, workspace: torch.Tensor = None, taps: bool = False,
                      events=None, coded=None, lora=None, gelu: bool = False, residual: torch.Tensor = None,
                      tuning: int = 0, readings=None):
    """Y = X W through the mixed decomposition (gelu=True: followed by the exact GELU, in the same kernels).
    residual: fp16 [M, N] added to the output as an fp16 addition, in the same kernels (may be `out` itself).
    taps: True for every intermediate, or a tuple of tap names.  With taps=True also returns a dict of the
    intermediates (outlier_mask, row_absmax, xq, acc, n_outliers, outlier_idx).
    coded=(codes, absmax, block): the activations arrive blockwise-coded; X is then the contiguous
    [M, K] fp16 buffer that receives the decoded values.
    lora=(A [r, K], B [N, r]) or (A, B, T_out [M, r]), fp16: adds the low-rank term of W' = W + B A.
    readings=(row_scale, W_master): the layer under the other readings (ROW_SCALE_* above; W_master: None or the
    original fp16 weights [K, N], whose rows then multiply the critical columns)."""
    _dev(X, torch.float16, "X")
    M, K = X.shape
    if K != pw.K or X.stride(1) != 1:
        raise Mmd8Error("X must be [M, %d] with unit stride along K" % pw.K)
    if coded is not None and not X.is_contiguous():
        raise Mmd8Error("the buffer for the decoded activations must be contiguous")
    N = pw.N
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=X.device)
    if readings is not None and (coded is not None or lora is not None):
        raise Mmd8Error("the alternative readings cannot be combined with coded activations or an adapter in one call")
    if coded is not None and lora is not None:
        raise Mmd8Error("coded activations and an adapter cannot be combined in one call")
    if gelu and (coded is not None or lora is not None):
        raise Mmd8Error("the activation cannot be combined with coded activations or an adapter in one call")
    if residual is not None:
        if gelu or coded is not None or lora is not None:
            raise Mmd8Error("the residual cannot be combined with an activation, coded activations or an adapter in one call")
        _dev(residual, torch.float16, "residual")
        if residual.shape != (M, N) or residual.stride(1) != 1:
            raise Mmd8Error("residual must be [M, N] with unit stride along N")
    if workspace is None:
        workspace = linear_workspace(M, K, N, X.device, lora[0].shape[0] if lora is not None else 0)
    tp, tensors = None, None
    if events is not None:                      # (begin, gemm_begin, gemm_end[, prep_mid]) hipEvent_t handles as ints
        tp = DebugTaps(event_begin=events[0], event_gemm_begin=events[1], event_gemm_end=events[2],
                       event_prep_mid=events[3] if len(events) > 3 else None)
    if taps:
        tensors = _taps(M, K, N, X.device, None if taps is True else tuple(taps))
        tp = DebugTaps(**{k: v.data_ptr() for k, v in tensors.items()})
    if tuning:                                  # kernel choice of this call (TUNE_* above)
        tp = tp if tp is not None else DebugTaps()
        tp.tuning = int(tuning)
    if coded is not None:
        codes, absmax, block = coded
        _dev(codes, torch.uint8, "codes")
        _dev(absmax, torch.float32, "absmax")
        _check(lib().mmd8_mixed_int8_linear_from_codes(
            codes.data_ptr(), absmax.data_ptr(), int(block), M, K, X.data_ptr(), pw.blob.data_ptr(),
            pw.layout, pw.col_absmax.data_ptr(), N, bias.data_ptr() if bias is not None else None, float(tau), out.data_ptr(),
            out.stride(0) if M > 0 else N, workspace.data_ptr(), workspace.numel(),
            ctypes.byref(tp) if tp is not None else None, _stream()))
        return (out, tensors) if taps else out
    if lora is not None:
        A, B = lora[0], lora[1]
        T_out = lora[2] if len(lora) > 2 else None
        _dev(A, torch.float16, "lora A")
        _dev(B, torch.float16, "lora B")
        r = A.shape[0]
        if A.shape != (r, K) or B.shape != (N, r) or not (A.is_contiguous() and B.is_contiguous()):
            raise Mmd8Error("adapter factors must be contiguous A [r, %d] and B [%d, r]" % (K, N))
        if T_out is not None and not (T_out.is_cuda and T_out.dtype == torch.float16 and T_out.shape == (M, r)
                                      and T_out.is_contiguous()):
            raise Mmd8Error("T_out must be a contiguous GPU fp16 tensor [M, r]")
        _check(lib().mmd8_mixed_int8_linear_lora(
            X.data_ptr(), M, K, X.stride(0) if M > 0 else K, pw.blob.data_ptr(), pw.layout, pw.col_absmax.data_ptr(), N,
            bias.data_ptr() if bias is not None else None, float(tau), A.data_ptr(), B.data_ptr(), int(r),
            T_out.data_ptr() if T_out is not None else None, out.data_ptr(), out.stride(0) if M > 0 else N,
            workspace.data_ptr(), workspace.numel(), ctypes.byref(tp) if tp is not None else None, _stream()))
        return (out, tensors) if taps else out
    if readings is not None:
        if gelu or residual is not None:
            raise Mmd8Error("the alternative readings cannot be combined with an activation or a residual in one call")
        row_scale, Wm = readings
        rd = Readings(int(row_scale), None, 0)
        if Wm is not None:
            _dev(Wm, torch.float16, "W_master")
            if Wm.shape != (K, N) or Wm.stride(1) != 1:
                raise Mmd8Error("W_master must be [K, N] with unit stride along N")
            rd = Readings(int(row_scale), Wm.data_ptr(), Wm.stride(0))
        _check(lib().mmd8_mixed_int8_linear_readings(
            X.data_ptr(), M, K, X.stride(0) if M > 0 else K, pw.blob.data_ptr(), pw.layout, pw.col_absmax.data_ptr(), N,
            bias.data_ptr() if bias is not None else None, float(tau), ctypes.byref(rd), out.data_ptr(),
            out.stride(0) if M > 0 else N, workspace.data_ptr(), workspace.numel(),
            ctypes.byref(tp) if tp is not None else None, _stream()))
        return (out, tensors) if taps else out
    if residual is not None:
        _check(lib().mmd8_mixed_int8_linear_residual(
            X.data_ptr(), M, K, X.stride(0) if M > 0 else K, pw.blob.data_ptr(), pw.layout, pw.col_absmax.data_ptr(), N,
            bias.data_ptr() if bias is not None else None, float(tau), residual.data_ptr(),
            residual.stride(0) if M > 0 else N, out.data_ptr(), out.stride(0) if M > 0 else N,
            workspace.data_ptr(), workspace.numel(), ctypes.byref(tp) if tp is not None else None, _stream()))
        return (out, tensors) if taps else out
    fn = lib().mmd8_mixed_int8_linear_gelu if gelu else lib().mmd8_mixed_int8_linear
    _check(fn(
        X.data_ptr(), M, K, X.stride(0) if M > 0 else K, pw.blob.data_ptr(), pw.layout, pw.col_absmax.data_ptr(), N,
        bias.data_ptr() if bias is not None else None, float(tau), out.data_ptr(), out.stride(0) if M > 0 else N,
        workspace.data_ptr(), workspace.numel(), ctypes.byref(tp) if tp is not None else None, _stream()))
    return (out, tensors) if taps else out


STATIC_WORKSPACE_BYTES = 32 << 20


def mixed_int8_linear_static(X: torch.Tensor, pw: PackedWeight, tau: float, out: torch.Tensor, bias: torch.Tensor = None,
                             taps: bool = False):
    """mixed_int8_linear without a workspace argument (the library's own device array serves as one): for callers
    that cannot allocate.  `out` must be given; nothing is allocated here unless taps are asked for."""
    _dev(X, torch.float16, "X")
    _dev(out, torch.float16, "out")
    M, K = X.shape
    if K != pw.K or X.stride(1) != 1:
        raise Mmd8Error("X must be [M, %d] with unit stride along K" % pw.K)
    N = pw.N
    if out.shape != (M, N) or out.stride(1) != 1:
        raise Mmd8Error("out must be [M, N] with unit stride along N")
    tensors = _taps(M, K, N, X.device) if taps else None
    tp = DebugTaps(**{k: v.data_ptr() for k, v in tensors.items()}) if taps else None
    _check(lib().mmd8_mixed_int8_linear_static(
        X.data_ptr(), M, K, X.stride(0) if M > 0 else K, pw.blob.data_ptr(), pw.layout, pw.col_absmax.data_ptr(), N,
        bias.data_ptr() if bias is not None else None, float(tau), out.data_ptr(), out.stride(0) if M > 0 else N,
        ctypes.byref(tp) if tp is not None else None, _stream()))
    return (out, tensors) if taps else out
