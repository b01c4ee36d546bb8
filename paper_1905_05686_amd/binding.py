"""ctypes binding of liblrbi.so.  Function names match include/lrbi.h without the
`lrbi_` prefix.  Device buffers are torch tensors (PyTorch is used for device
memory and streams only); host buffers are numpy arrays."""
from __future__ import annotations

import ctypes
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "liblrbi.so")
_lib = None

F32, F16, BF16 = 0, 1, 2
FLAG_PATH_VALU = 0x1
FLAG_PATH_MFMA = 0x2
FLAG_PATH_STREAM = 0x3
FLAG_DECODE_GENERIC = 0x00100000


def flag_splitk(s: int) -> int:
    return (int(s) & 0xFF) << 8


def flag_tile(t: int) -> int:
    return (int(t) & 0xF) << 16


class LrbiError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %d (%s)" % (where, status, strerror(status)))


class Desc(ctypes.Structure):
    """Mirror of lrbi_desc: W is m x n, tiles r x c, rank k."""
    _fields_ = [("m", ctypes.c_int64), ("n", ctypes.c_int64), ("r", ctypes.c_int32), ("c", ctypes.c_int32),
                ("k", ctypes.c_int32), ("flags", ctypes.c_uint32)]

    def __init__(self, m, n, r, c, k, flags=0):
        super().__init__(int(m), int(n), int(r), int(c), int(k), int(flags))

    def with_flags(self, flags: int) -> "Desc":
        return Desc(self.m, self.n, self.r, self.c, self.k, flags)

    @property
    def tiles(self) -> int:
        return (-(-self.m // self.r)) * (-(-self.n // self.c))


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load liblrbi.so.  Raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError("liblrbi.so is missing at %s: build it with `python -m paper_1905_05686_amd.build` "
                           "(there is no CPU fallback)" % _LIB_PATH)
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i64, u64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_uint64, ctypes.c_int32
    pd = ctypes.POINTER(Desc)
    pu64 = ctypes.POINTER(ctypes.c_uint64)
    lib.lrbi_strerror.argtypes = [ctypes.c_int]
    lib.lrbi_strerror.restype = ctypes.c_char_p
    lib.lrbi_index_bits.argtypes = [pd, pu64, pu64, pu64, pu64]
    lib.lrbi_csr_bits.argtypes = [u64, i64, i32, i32, pu64]
    lib.lrbi_pack_factors.argtypes = [pd, vp, vp, vp, vp]
    lib.lrbi_pack_factors_ranked.argtypes = [pd, vp, vp, vp, vp, vp]
    lib.lrbi_index_bits_ranked.argtypes = [pd, vp, pu64]
    lib.lrbi_unpack_mask.argtypes = [pd, vp, i64, vp]
    lib.lrbi_decode_mask.argtypes = [pd, vp, vp, vp, i64, vp]
    lib.lrbi_masked_gemm_workspace_bytes.argtypes = [pd, ctypes.c_int, i64, pu64]
    lib.lrbi_masked_gemm.argtypes = [pd, ctypes.c_int, vp, i64, vp, vp, vp, i64, i64, vp, i64, vp, u64, vp]
    lib.lrbi_decode_and_gemm.argtypes = [pd, ctypes.c_int, vp, i64, vp, vp, vp, i64, i64, vp, i64, vp, i64, vp, u64, vp]
    lib.lrbi_masked_conv3x3_workspace_bytes.argtypes = [pd, ctypes.c_int, i64, i64, i64, pu64]
    lib.lrbi_masked_conv3x3.argtypes = [pd, ctypes.c_int, vp, i64, vp, vp, vp, i64, i64, i64, i64, vp, i64, vp, u64, vp]
    lib.lrbi_masked_gemm_static.argtypes = [pd, ctypes.c_int, vp, i64, vp, vp, vp, i64, i64, vp, i64, vp]
    lib.lrbi_threshold_eval.argtypes = [pd, ctypes.c_int, vp, i64, ctypes.c_float, ctypes.c_int32, ctypes.c_float, vp, vp, vp, vp, vp, vp, vp, vp, vp, u64,
                                        vp]
    lib.lrbi_threshold_eval_workspace_bytes.argtypes = [pd, pu64]
    lib.lrbi_search_thresholds.argtypes = [pd, ctypes.c_int, vp, i64, ctypes.c_float, ctypes.c_int32, ctypes.c_float, vp, vp, ctypes.c_double,
                                           ctypes.POINTER(ctypes.c_double), i32, i32, i64, vp, vp, vp, vp, vp, vp, vp, u64,
                                           vp]
    lib.lrbi_search_workspace_bytes.argtypes = [pd, pu64]
    lib.lrbi_masked_gemm_t_workspace_bytes.argtypes = [pd, ctypes.c_int, i64, pu64]
    lib.lrbi_masked_gemm_t.argtypes = [pd, ctypes.c_int, vp, i64, vp, vp, vp, i64, i64, vp, i64, vp, u64, vp]
    lib.lrbi_masked_grad.argtypes = [pd, ctypes.c_int, vp, i64, vp, i64, i64, vp, vp, vp, i64, vp]
    lib.lrbi_lstm_step_workspace_bytes.argtypes = [pd, ctypes.c_int, i64, pu64]
    lib.lrbi_nmf_workspace_bytes.argtypes = [pd, pu64]
    lib.lrbi_nmf.argtypes = [pd, ctypes.c_int, vp, i64, i32, ctypes.c_float, ctypes.c_float, vp, vp, i32, ctypes.c_float,
                             vp, u64, vp]
    lib.lrbi_lstm_step.argtypes = [pd, ctypes.c_int, vp, i64, vp, vp, vp, i64, i64, vp, i64, vp, i64, vp, i64, vp, u64, vp]
    for name in ("lrbi_index_bits", "lrbi_index_bits_ranked", "lrbi_pack_factors_ranked", "lrbi_csr_bits",
                 "lrbi_pack_factors", "lrbi_unpack_mask", "lrbi_decode_mask",
                 "lrbi_masked_gemm_workspace_bytes", "lrbi_masked_gemm", "lrbi_masked_gemm_static", "lrbi_threshold_eval",
                 "lrbi_threshold_eval_workspace_bytes", "lrbi_search_thresholds", "lrbi_search_workspace_bytes",
                 "lrbi_masked_gemm_t_workspace_bytes", "lrbi_masked_gemm_t", "lrbi_masked_grad",
                 "lrbi_lstm_step_workspace_bytes", "lrbi_lstm_step", "lrbi_nmf_workspace_bytes", "lrbi_nmf"):
        getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def strerror(status: int) -> str:
    return load_library().lrbi_strerror(int(status)).decode()


def _check(status: int, where: str):
    if status != 0:
        raise LrbiError(status, where)


def index_bits(desc: Desc) -> dict:
    """lrbi_index_bits: factor bits, dense bitmask bits and packed buffer sizes."""
    a, b, c, d = (ctypes.c_uint64() for _ in range(4))
    _check(load_library().lrbi_index_bits(ctypes.byref(desc), ctypes.byref(a), ctypes.byref(b), ctypes.byref(c),
                                          ctypes.byref(d)), "lrbi_index_bits")
    return {"lrbi_bits": a.value, "dense_bits": b.value, "packed_ip_bytes": c.value, "packed_iz_bytes": d.value}


def csr_bits(nnz: int, m: int, idx_bits: int = 16, ptr_bits: int = 32) -> int:
    out = ctypes.c_uint64()
    _check(load_library().lrbi_csr_bits(int(nnz), int(m), int(idx_bits), int(ptr_bits), ctypes.byref(out)),
           "lrbi_csr_bits")
    return out.value


def index_bits_ranked(desc: Desc, tile_rank) -> int:
    """lrbi_index_bits_ranked: factor bits with a rank per tile (int32 [T])."""
    tile_rank = np.ascontiguousarray(tile_rank, dtype=np.int32)
    if tile_rank.shape != (desc.tiles,):
        raise ValueError("tile_rank must have one entry per tile")
    out = ctypes.c_uint64()
    _check(load_library().lrbi_index_bits_ranked(ctypes.byref(desc), tile_rank.ctypes.data, ctypes.byref(out)),
           "lrbi_index_bits_ranked")
    return out.value


def pack_factors(desc: Desc, Ip01: np.ndarray, Iz01: np.ndarray, tile_rank=None):
    """lrbi_pack_factors / lrbi_pack_factors_ranked: uint8 0/1 factors [T,r,k], [T,k,c] -> packed host arrays
    (uint32 [T*r, ceil(k/32)], uint64 [T*k, ceil(c/64)]); tile_rank int32 [T] (optional) = rank of every tile."""
    Ip01 = np.ascontiguousarray(Ip01, dtype=np.uint8)
    Iz01 = np.ascontiguousarray(Iz01, dtype=np.uint8)
    T = desc.tiles
    if Ip01.shape != (T, desc.r, desc.k) or Iz01.shape != (T, desc.k, desc.c):
        raise ValueError("factor shapes do not match the descriptor")
    sizes = index_bits(desc)
    ip = np.empty((T * desc.r, sizes["packed_ip_bytes"] // (4 * T * desc.r)), dtype=np.uint32)
    iz = np.empty((T * desc.k, sizes["packed_iz_bytes"] // (8 * T * desc.k)), dtype=np.uint64)
    if tile_rank is not None:
        tile_rank = np.ascontiguousarray(tile_rank, dtype=np.int32)
        if tile_rank.shape != (T,):
            raise ValueError("tile_rank must have one entry per tile")
        _check(load_library().lrbi_pack_factors_ranked(ctypes.byref(desc), tile_rank.ctypes.data, Ip01.ctypes.data,
                                                       Iz01.ctypes.data, ip.ctypes.data, iz.ctypes.data),
               "lrbi_pack_factors_ranked")
        return ip, iz
    _check(load_library().lrbi_pack_factors(ctypes.byref(desc), Ip01.ctypes.data, Iz01.ctypes.data, ip.ctypes.data,
                                            iz.ctypes.data), "lrbi_pack_factors")
    return ip, iz


def unpack_mask(desc: Desc, mask_bytes: np.ndarray) -> np.ndarray:
    """lrbi_unpack_mask: packed host mask [m, pitch] (uint8) -> uint8 0/1 [m, n]."""
    mask_bytes = np.ascontiguousarray(mask_bytes, dtype=np.uint8)
    if mask_bytes.ndim != 2 or mask_bytes.shape[0] != desc.m:
        raise ValueError("mask must be [m, pitch_bytes]")
    out = np.empty((desc.m, desc.n), dtype=np.uint8)
    _check(load_library().lrbi_unpack_mask(ctypes.byref(desc), mask_bytes.ctypes.data, mask_bytes.shape[1],
                                           out.ctypes.data), "lrbi_unpack_mask")
    return out


def _stream_ptr(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dev_ptr(t, what):
    if not t.is_cuda:
        raise ValueError("%s must be a device tensor" % what)
    return ctypes.c_void_p(t.data_ptr())


def default_pitch(n: int) -> int:
    return ((n + 127) // 128) * 16


def decode_mask(desc: Desc, dIp, dIz, out=None, pitch_bytes=None, stream=None):
    """lrbi_decode_mask: packed device factors -> packed device mask [m, pitch] (uint8)."""
    import torch
    if pitch_bytes is None:
        pitch_bytes = out.shape[1] if out is not None else default_pitch(desc.n)
    if out is None:
        out = torch.empty((desc.m, pitch_bytes), dtype=torch.uint8, device=dIp.device)
    if out.dtype != torch.uint8 or not out.is_contiguous() or out.shape != (desc.m, pitch_bytes):
        raise ValueError("out must be a contiguous uint8 [m, pitch_bytes] tensor")
    _check(load_library().lrbi_decode_mask(ctypes.byref(desc), _dev_ptr(dIp, "Ip"), _dev_ptr(dIz, "Iz"),
                                           _dev_ptr(out, "mask"), int(pitch_bytes), _stream_ptr(stream)),
           "lrbi_decode_mask")
    return out


def _dtype_code(t):
    import torch
    return {torch.float32: F32, torch.float16: F16, torch.bfloat16: BF16}[t.dtype]


def masked_gemm_workspace_bytes(desc: Desc, dtype_code: int, N: int) -> int:
    out = ctypes.c_uint64()
    _check(load_library().lrbi_masked_gemm_workspace_bytes(ctypes.byref(desc), int(dtype_code), int(N),
                                                           ctypes.byref(out)), "lrbi_masked_gemm_workspace_bytes")
    return out.value


def masked_gemm(desc: Desc, W, dIp, dIz, X, out=None, workspace=None, stream=None):
    """lrbi_masked_gemm: Y = (W o decode(Ip, Iz)) X.  W [m, n], X [n, N] (or [n]),
    row-major device tensors of one dtype; rows may be padded (stride(0) >= width)."""
    import torch
    squeeze = X.dim() == 1
    if squeeze:
        X = X.unsqueeze(1)
    if W.dim() != 2 or X.dim() != 2 or W.shape != (desc.m, desc.n) or X.shape[0] != desc.n:
        raise ValueError("shape mismatch")
    if W.stride(1) != 1 or (X.shape[1] > 1 and X.stride(1) != 1) or W.dtype != X.dtype:
        raise ValueError("W and X must be row-major tensors of the same dtype")
    N = X.shape[1]
    if out is None:
        out = torch.empty((desc.m, N), dtype=W.dtype, device=W.device)
    if out.shape != (desc.m, N) or out.dtype != W.dtype or (N > 1 and out.stride(1) != 1):
        raise ValueError("bad out tensor")
    ws_ptr, ws_bytes = ctypes.c_void_p(0), 0
    if workspace is not None:
        ws_ptr, ws_bytes = _dev_ptr(workspace, "workspace"), workspace.numel() * workspace.element_size()
    _check(load_library().lrbi_masked_gemm(
        ctypes.byref(desc), _dtype_code(W), _dev_ptr(W, "W"), W.stride(0), _dev_ptr(dIp, "Ip"), _dev_ptr(dIz, "Iz"),
        _dev_ptr(X, "X"), X.stride(0), N, _dev_ptr(out, "Y"), out.stride(0), ws_ptr, ws_bytes, _stream_ptr(stream)),
        "lrbi_masked_gemm")
    return out[:, 0] if squeeze else out


def decode_and_gemm(desc: Desc, W, dIp, dIz, X, out=None, mask=None, pitch_bytes=None, workspace=None, stream=None):
    """lrbi_decode_and_gemm: the packed mask [m, pitch] (uint8) and Y = (W o mask) X from one call; arguments as
    for decode_mask and masked_gemm.  Returns (mask, Y)."""
    import torch
    if W.dim() != 2 or X.dim() != 2 or W.shape != (desc.m, desc.n) or X.shape[0] != desc.n:
        raise ValueError("shape mismatch")
    if W.stride(1) != 1 or (X.shape[1] > 1 and X.stride(1) != 1) or W.dtype != X.dtype:
        raise ValueError("W and X must be row-major tensors of the same dtype")
    N = X.shape[1]
    if out is None:
        out = torch.empty((desc.m, N), dtype=W.dtype, device=W.device)
    if out.shape != (desc.m, N) or out.dtype != W.dtype or (N > 1 and out.stride(1) != 1):
        raise ValueError("bad out tensor")
    if pitch_bytes is None:
        pitch_bytes = mask.shape[1] if mask is not None else default_pitch(desc.n)
    if mask is None:
        mask = torch.empty((desc.m, pitch_bytes), dtype=torch.uint8, device=W.device)
    if mask.dtype != torch.uint8 or not mask.is_contiguous() or mask.shape != (desc.m, pitch_bytes):
        raise ValueError("mask must be a contiguous uint8 [m, pitch_bytes] tensor")
    ws_ptr, ws_bytes = ctypes.c_void_p(0), 0
    if workspace is not None:
        ws_ptr, ws_bytes = _dev_ptr(workspace, "workspace"), workspace.numel() * workspace.element_size()
    _check(load_library().lrbi_decode_and_gemm(
        ctypes.byref(desc), _dtype_code(W), _dev_ptr(W, "W"), W.stride(0), _dev_ptr(dIp, "Ip"), _dev_ptr(dIz, "Iz"),
        _dev_ptr(X, "X"), X.stride(0), N, _dev_ptr(out, "Y"), out.stride(0), _dev_ptr(mask, "mask"), int(pitch_bytes),
        ws_ptr, ws_bytes, _stream_ptr(stream)), "lrbi_decode_and_gemm")
    return mask, out


def masked_conv3x3_workspace_bytes(desc: Desc, dtype_code: int, batch: int, H: int, Wd: int) -> int:
    out = ctypes.c_uint64()
    _check(load_library().lrbi_masked_conv3x3_workspace_bytes(ctypes.byref(desc), int(dtype_code), int(batch), int(H),
                                                              int(Wd), ctypes.byref(out)),
           "lrbi_masked_conv3x3_workspace_bytes")
    return out.value


def masked_conv3x3(desc: Desc, W, dIp, dIz, act_padded, out=None, workspace=None, stream=None):
    """lrbi_masked_conv3x3: Y = (W o decode(Ip, Iz)) X for a 3 x 3, padding-1 convolution, X gathered from the
    activation.  W [m, 9 * cin] with column (kh * 3 + kw) * cin + ci; act_padded [batch, H + 2, Wd + 2, cin]
    contiguous with a zero border; returns Y [m, batch * H * Wd]."""
    import torch
    if act_padded.dim() != 4 or not act_padded.is_contiguous() or act_padded.dtype != W.dtype:
        raise ValueError("act_padded must be a contiguous [batch, H + 2, Wd + 2, cin] tensor of W's dtype")
    batch, H, Wd, cin = act_padded.shape[0], act_padded.shape[1] - 2, act_padded.shape[2] - 2, act_padded.shape[3]
    if W.dim() != 2 or W.shape != (desc.m, desc.n) or W.stride(1) != 1:
        raise ValueError("shape mismatch")
    N = batch * H * Wd
    if out is None:
        out = torch.empty((desc.m, N), dtype=W.dtype, device=W.device)
    if out.shape != (desc.m, N) or out.dtype != W.dtype or out.stride(1) != 1:
        raise ValueError("bad out tensor")
    ws_ptr, ws_bytes = ctypes.c_void_p(0), 0
    if workspace is not None:
        ws_ptr, ws_bytes = _dev_ptr(workspace, "workspace"), workspace.numel() * workspace.element_size()
    _check(load_library().lrbi_masked_conv3x3(
        ctypes.byref(desc), _dtype_code(W), _dev_ptr(W, "W"), W.stride(0), _dev_ptr(dIp, "Ip"), _dev_ptr(dIz, "Iz"),
        _dev_ptr(act_padded, "act"), batch, H, Wd, cin, _dev_ptr(out, "Y"), out.stride(0), ws_ptr, ws_bytes,
        _stream_ptr(stream)), "lrbi_masked_conv3x3")
    return out


STATIC_SCRATCH_BYTES = 32 * 1024 * 1024


def masked_gemm_static(desc: Desc, W, dIp, dIz, X, out, stream=None):
    """lrbi_masked_gemm_static: as masked_gemm, with the library's own static scratch array instead of a workspace.
    `out` [m, N] must be given: the call itself allocates nothing."""
    if W.dim() != 2 or X.dim() != 2 or W.shape != (desc.m, desc.n) or X.shape[0] != desc.n:
        raise ValueError("shape mismatch")
    if W.stride(1) != 1 or (X.shape[1] > 1 and X.stride(1) != 1) or W.dtype != X.dtype:
        raise ValueError("W and X must be row-major tensors of the same dtype")
    N = X.shape[1]
    if out.shape != (desc.m, N) or out.dtype != W.dtype or (N > 1 and out.stride(1) != 1):
        raise ValueError("bad out tensor")
    _check(load_library().lrbi_masked_gemm_static(
        ctypes.byref(desc), _dtype_code(W), _dev_ptr(W, "W"), W.stride(0), _dev_ptr(dIp, "Ip"), _dev_ptr(dIz, "Iz"),
        _dev_ptr(X, "X"), X.stride(0), N, _dev_ptr(out, "Y"), out.stride(0), _stream_ptr(stream)),
        "lrbi_masked_gemm_static")
    return out


def threshold_eval_workspace_bytes(desc: Desc) -> int:
    out = ctypes.c_uint64()
    _check(load_library().lrbi_threshold_eval_workspace_bytes(ctypes.byref(desc), ctypes.byref(out)),
           "lrbi_threshold_eval_workspace_bytes")
    return out.value


def threshold_eval(desc: Desc, W, w_threshold: float, Mp, Mz, Tp, Tz, want_factors: bool = False, out=None,
                   workspace=None, stream=None, method: int = 1, amplify: float = 1.0):
    """lrbi_threshold_eval: one candidate of Algorithm 1 for every tile.  W [m, n] (f32 / f16 / bf16),
    Mp [T, r, k], Mz [T, k, c], Tp, Tz [T] float32 device tensors.  Returns (kept int64 [T], cost float64 [T])
    and, with want_factors, also the packed factors (Ip int32 [T*r, ipw], Iz int32 [T*k, izw]).
    `out` = (kept, cost) reuses existing result tensors; `workspace` = device scratch of at least
    threshold_eval_workspace_bytes(desc) bytes (optional).  method / amplify: the magnitude manipulation the
    cost is summed over (1 none, 2 squared, 3 amplified), as given to nmf()."""
    import torch
    T = desc.tiles
    if W.dim() != 2 or W.shape != (desc.m, desc.n) or W.stride(1) != 1:
        raise ValueError("W must be a row-major [m, n] tensor")
    for t, shape in ((Mp, (T, desc.r, desc.k)), (Mz, (T, desc.k, desc.c)), (Tp, (T,)), (Tz, (T,))):
        if t.dtype != torch.float32 or tuple(t.shape) != shape or not t.is_contiguous():
            raise ValueError("factor / threshold tensors must be contiguous float32 of shape %s" % (shape,))
    if out is not None:
        kept, cost = out
        if kept.dtype != torch.int64 or cost.dtype != torch.float64 or kept.numel() != T or cost.numel() != T:
            raise ValueError("out must be (int64 [T], float64 [T])")
    else:
        kept = torch.empty(T, dtype=torch.int64, device=W.device)
        cost = torch.empty(T, dtype=torch.float64, device=W.device)
    ip = iz = None
    if want_factors:
        ip = torch.empty((T * desc.r, (desc.k + 31) // 32), dtype=torch.int32, device=W.device)
        iz = torch.empty((T * desc.k, 2 * ((desc.c + 63) // 64)), dtype=torch.int32, device=W.device)
    _check(load_library().lrbi_threshold_eval(
        ctypes.byref(desc), _dtype_code(W), _dev_ptr(W, "W"), W.stride(0), float(w_threshold), int(method),
        float(amplify), _dev_ptr(Mp, "Mp"), _dev_ptr(Mz, "Mz"), _dev_ptr(Tp, "Tp"), _dev_ptr(Tz, "Tz"), _dev_ptr(ip, "Ip") if want_factors else None,
        _dev_ptr(iz, "Iz") if want_factors else None, _dev_ptr(kept, "kept"), _dev_ptr(cost, "cost"),
        _dev_ptr(workspace, "workspace") if workspace is not None else None,
        workspace.numel() * workspace.element_size() if workspace is not None else 0,
        _stream_ptr(stream)), "lrbi_threshold_eval")
    return (kept, cost, ip, iz) if want_factors else (kept, cost)


def search_workspace_bytes(desc: Desc) -> int:
    out = ctypes.c_uint64()
    _check(load_library().lrbi_search_workspace_bytes(ctypes.byref(desc), ctypes.byref(out)),
           "lrbi_search_workspace_bytes")
    return out.value


def search_thresholds(desc: Desc, W, w_threshold: float, Mp, Mz, target_sparsity: float, sp_values, steps: int,
                      tolerance: int, want_factors: bool = False, workspace=None, stream=None, method: int = 1,
                      amplify: float = 1.0):
    """lrbi_search_thresholds: the threshold search of Algorithm 1 for every tile.  W [m, n] (f32 / f16 / bf16),
    Mp [T, r, k], Mz [T, k, c] float32 device tensors; sp_values a host sequence of floats.  Returns
    (Tp float32 [T], Tz float32 [T], kept int64 [T], cost float64 [T]) and, with want_factors, also the packed
    factors (Ip int32 [T*r, ipw], Iz int32 [T*k, izw]) converted with the winning thresholds.  `workspace` =
    device scratch of at least search_workspace_bytes(desc) bytes (allocated here when None)."""
    import torch
    T = desc.tiles
    if W.dim() != 2 or W.shape != (desc.m, desc.n) or W.stride(1) != 1:
        raise ValueError("W must be a row-major [m, n] tensor")
    for t, shape in ((Mp, (T, desc.r, desc.k)), (Mz, (T, desc.k, desc.c))):
        if t.dtype != torch.float32 or tuple(t.shape) != shape or not t.is_contiguous():
            raise ValueError("factor tensors must be contiguous float32 of shape %s" % (shape,))
    if workspace is None:
        workspace = torch.empty(search_workspace_bytes(desc), dtype=torch.uint8, device=W.device)
    sp = (ctypes.c_double * len(sp_values))(*[float(v) for v in sp_values])
    Tp = torch.empty(T, dtype=torch.float32, device=W.device)
    Tz = torch.empty(T, dtype=torch.float32, device=W.device)
    kept = torch.empty(T, dtype=torch.int64, device=W.device)
    cost = torch.empty(T, dtype=torch.float64, device=W.device)
    ip = iz = None
    if want_factors:
        ip = torch.empty((T * desc.r, (desc.k + 31) // 32), dtype=torch.int32, device=W.device)
        iz = torch.empty((T * desc.k, 2 * ((desc.c + 63) // 64)), dtype=torch.int32, device=W.device)
    _check(load_library().lrbi_search_thresholds(
        ctypes.byref(desc), _dtype_code(W), _dev_ptr(W, "W"), W.stride(0), float(w_threshold), int(method),
        float(amplify), _dev_ptr(Mp, "Mp"), _dev_ptr(Mz, "Mz"), float(target_sparsity), sp, len(sp_values), int(steps), int(tolerance), _dev_ptr(Tp, "Tp"),
        _dev_ptr(Tz, "Tz"), _dev_ptr(kept, "kept"), _dev_ptr(cost, "cost"), _dev_ptr(ip, "Ip") if want_factors else None,
        _dev_ptr(iz, "Iz") if want_factors else None, _dev_ptr(workspace, "workspace"),
        workspace.numel() * workspace.element_size(), _stream_ptr(stream)), "lrbi_search_thresholds")
    return (Tp, Tz, kept, cost, ip, iz) if want_factors else (Tp, Tz, kept, cost)


def masked_gemm_t_workspace_bytes(desc: Desc, dtype_code: int, N: int) -> int:
    out = ctypes.c_uint64()
    _check(load_library().lrbi_masked_gemm_t_workspace_bytes(ctypes.byref(desc), int(dtype_code), int(N),
                                                             ctypes.byref(out)), "lrbi_masked_gemm_t_workspace_bytes")
    return out.value


def masked_gemm_t(desc: Desc, W, dIp, dIz, dY, out=None, workspace=None, stream=None):
    """lrbi_masked_gemm_t: dX = (W o decode(Ip, Iz))^T dY.  W [m, n], dY [m, N] row-major device tensors of one
    dtype (rows may be padded); returns dX [n, N]."""
    import torch
    if W.dim() != 2 or dY.dim() != 2 or W.shape != (desc.m, desc.n) or dY.shape[0] != desc.m:
        raise ValueError("shape mismatch")
    if W.stride(1) != 1 or (dY.shape[1] > 1 and dY.stride(1) != 1) or W.dtype != dY.dtype:
        raise ValueError("W and dY must be row-major tensors of the same dtype")
    N = dY.shape[1]
    if out is None:
        out = torch.empty((desc.n, N), dtype=W.dtype, device=W.device)
    if out.shape != (desc.n, N) or out.dtype != W.dtype or (N > 1 and out.stride(1) != 1):
        raise ValueError("bad out tensor")
    ws_ptr, ws_bytes = ctypes.c_void_p(0), 0
    if workspace is not None:
        ws_ptr, ws_bytes = _dev_ptr(workspace, "workspace"), workspace.numel() * workspace.element_size()
    _check(load_library().lrbi_masked_gemm_t(
        ctypes.byref(desc), _dtype_code(W), _dev_ptr(W, "W"), W.stride(0), _dev_ptr(dIp, "Ip"), _dev_ptr(dIz, "Iz"),
        _dev_ptr(dY, "dY"), dY.stride(0), N, _dev_ptr(out, "dX"), out.stride(0), ws_ptr, ws_bytes,
        _stream_ptr(stream)), "lrbi_masked_gemm_t")
    return out


def masked_grad(desc: Desc, dY, X, dIp, dIz, out=None, stream=None):
    """lrbi_masked_grad: dW = (dY X^T) o decode(Ip, Iz).  dY [m, N], X [n, N] row-major device tensors of one
    dtype (rows may be padded); returns dW [m, n] with exact zeros at pruned weights."""
    import torch
    if dY.dim() != 2 or X.dim() != 2 or dY.shape[0] != desc.m or X.shape[0] != desc.n or dY.shape[1] != X.shape[1]:
        raise ValueError("shape mismatch")
    N = dY.shape[1]
    if (N > 1 and (dY.stride(1) != 1 or X.stride(1) != 1)) or dY.dtype != X.dtype:
        raise ValueError("dY and X must be row-major tensors of the same dtype")
    if out is None:
        out = torch.empty((desc.m, desc.n), dtype=dY.dtype, device=dY.device)
    if out.shape != (desc.m, desc.n) or out.dtype != dY.dtype or out.stride(1) != 1:
        raise ValueError("bad out tensor")
    _check(load_library().lrbi_masked_grad(
        ctypes.byref(desc), _dtype_code(dY), _dev_ptr(dY, "dY"), dY.stride(0), _dev_ptr(X, "X"), X.stride(0), N,
        _dev_ptr(dIp, "Ip"), _dev_ptr(dIz, "Iz"), _dev_ptr(out, "dW"), out.stride(0), _stream_ptr(stream)),
        "lrbi_masked_grad")
    return out


def lstm_step_workspace_bytes(desc: Desc, dtype_code: int, B: int) -> int:
    out = ctypes.c_uint64()
    _check(load_library().lrbi_lstm_step_workspace_bytes(ctypes.byref(desc), int(dtype_code), int(B), ctypes.byref(out)),
           "lrbi_lstm_step_workspace_bytes")
    return out.value


def lstm_step(desc: Desc, W, dIp, dIz, XH, C, H1, H2=None, workspace=None, stream=None):
    """lrbi_lstm_step: one LSTM step on the masked gate matrix W [4H, n].  XH [n, B] (f16 / bf16), C [H, B] float32
    (updated in place), H1 (and H2, optional) [H, B] of W's dtype receive h; they may be row slices of the buffer XH
    lives in.  `workspace`: device scratch of at least lstm_step_workspace_bytes bytes (allocated here when None)."""
    import torch
    Hh = desc.m // 4
    B = XH.shape[1]
    if W.shape != (desc.m, desc.n) or XH.shape[0] != desc.n or C.shape != (Hh, B) or C.dtype != torch.float32:
        raise ValueError("shape mismatch")
    for t in (H1, H2):
        if t is not None and (t.shape != (Hh, B) or t.dtype != W.dtype or (B > 1 and t.stride(1) != 1)):
            raise ValueError("bad h output tensor")
    if W.stride(1) != 1 or (B > 1 and (XH.stride(1) != 1 or C.stride(1) != 1)) or XH.dtype != W.dtype:
        raise ValueError("row-major tensors of one dtype expected")
    if workspace is None:
        workspace = torch.empty(lstm_step_workspace_bytes(desc, _dtype_code(W), B), dtype=torch.uint8, device=W.device)
    _check(load_library().lrbi_lstm_step(
        ctypes.byref(desc), _dtype_code(W), _dev_ptr(W, "W"), W.stride(0), _dev_ptr(dIp, "Ip"), _dev_ptr(dIz, "Iz"),
        _dev_ptr(XH, "XH"), XH.stride(0), B, _dev_ptr(C, "C"), C.stride(0), _dev_ptr(H1, "H1"), H1.stride(0),
        _dev_ptr(H2, "H2") if H2 is not None else None, H2.stride(0) if H2 is not None else 0,
        _dev_ptr(workspace, "workspace"), workspace.numel() * workspace.element_size(), _stream_ptr(stream)),
        "lrbi_lstm_step")
    return H1


def nmf_workspace_bytes(desc: Desc) -> int:
    out = ctypes.c_uint64()
    _check(load_library().lrbi_nmf_workspace_bytes(ctypes.byref(desc), ctypes.byref(out)), "lrbi_nmf_workspace_bytes")
    return out.value


def nmf(desc: Desc, W, Mp, Mz, iters: int, eps: float = 1e-9, method: int = 1, w_threshold: float = 0.0,
        amplify: float = 1.0, workspace=None, stream=None):
    """lrbi_nmf: multiplicative updates of |W| ~ Mp Mz per tile, in place.  W [m, n] (f32 / f16 / bf16), Mp [T, r, k],
    Mz [T, k, c] contiguous float32 device tensors holding the starting point.  Returns (Mp, Mz)."""
    import torch
    T = desc.tiles
    if W.dim() != 2 or W.shape != (desc.m, desc.n) or W.stride(1) != 1:
        raise ValueError("W must be a row-major [m, n] tensor")
    for t, shape in ((Mp, (T, desc.r, desc.k)), (Mz, (T, desc.k, desc.c))):
        if t.dtype != torch.float32 or tuple(t.shape) != shape or not t.is_contiguous():
            raise ValueError("factor tensors must be contiguous float32 of shape %s" % (shape,))
    if workspace is None:
        workspace = torch.empty(nmf_workspace_bytes(desc), dtype=torch.uint8, device=W.device)
    _check(load_library().lrbi_nmf(
        ctypes.byref(desc), _dtype_code(W), _dev_ptr(W, "W"), W.stride(0), int(method), float(w_threshold), float(amplify),
        _dev_ptr(Mp, "Mp"), _dev_ptr(Mz, "Mz"), int(iters), float(eps), _dev_ptr(workspace, "workspace"),
        workspace.numel() * workspace.element_size(), _stream_ptr(stream)), "lrbi_nmf")
    return Mp, Mz
