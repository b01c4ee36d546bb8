"""C ABI: the library loads without a GPU, exports every symbol the header
declares, validates arguments before touching the GPU, and its host-only entry
points agree with independent numpy formulations.  CPU only."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_1905_05686_amd as lrbi
from oracle import lrbi_oracle as orc
import workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "lrbi.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lrbi_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = lrbi.load_library()
    syms = _declared_symbols()
    assert {"lrbi_decode_mask", "lrbi_masked_gemm", "lrbi_index_bits"} <= set(syms)
    for s in syms:
        assert hasattr(lib, s), s


def test_strerror_covers_all_codes():
    for code in range(0, -10, -1):
        assert lrbi.strerror(code) and "unknown lrbi status" not in lrbi.strerror(code)
    assert "unknown lrbi status" in lrbi.strerror(-99)


@pytest.mark.parametrize("name", ["C1", "C2", "C3a", "C4", "C5"])
def test_index_bits_matches_oracle(name):
    cfg = workloads.CONFIGS[name]
    d = lrbi.Desc(cfg.m, cfg.n, cfg.r, cfg.c, cfg.k)
    got = lrbi.index_bits(d)
    assert got["lrbi_bits"] == orc.index_bits(cfg.m, cfg.n, cfg.r, cfg.c, cfg.k)
    assert got["dense_bits"] == orc.dense_bits(cfg.m, cfg.n)
    assert got["packed_ip_bytes"] == cfg.tiles * cfg.r * 4 * ((cfg.k + 31) // 32)
    assert got["packed_iz_bytes"] == cfg.tiles * cfg.k * 8 * ((cfg.c + 63) // 64)
    assert lrbi.csr_bits(12345, cfg.m, 16, 32) == orc.csr_bits(12345, cfg.m, 16, 32)


def test_desc_validation():
    bad = [
        (lrbi.Desc(0, 8, 1, 1, 1), -2), (lrbi.Desc(8, 8, 0, 4, 1), -2), (lrbi.Desc(8, 8, 4, -3, 1), -2),
        (lrbi.Desc(8, 8, 4, 4, 0), -3), (lrbi.Desc(8, 8, 4, 4, 257), -3), (lrbi.Desc(8, 8, 4, 4, 1, 1 << 30), -9),
        (lrbi.Desc(8, 8, 4, 4, 1, 4), -9),  # path values beyond the three kernels
    ]
    for d, code in bad:
        with pytest.raises(lrbi.LrbiError) as e:
            lrbi.index_bits(d)
        assert e.value.status == code
    # tiles need not divide the matrix: the last tile row / column is cut off at the edge
    assert lrbi.Desc(8, 8, 3, 4, 1).tiles == 6 and lrbi.index_bits(lrbi.Desc(8, 8, 3, 4, 1))["lrbi_bits"] == 2 * 8 + 3 * 8


def test_edge_tiles_and_ranks_host_side():
    """Sizes and packing for cut-off edge tiles and per-tile ranks against the oracle / numpy."""
    rng = np.random.default_rng(5)
    for (m, n, r, c, k) in [(70, 90, 32, 40, 5), (577, 1000, 576, 512, 145), (7, 9, 3, 4, 2)]:
        d = lrbi.Desc(m, n, r, c, k)
        T = d.tiles
        assert T == orc.num_tiles(m, n, r, c)
        got = lrbi.index_bits(d)
        assert got["lrbi_bits"] == orc.index_bits(m, n, r, c, k)
        assert got["packed_ip_bytes"] == T * r * 4 * ((k + 31) // 32)
        rank = rng.integers(0, k + 1, size=T).astype(np.int32)
        assert lrbi.index_bits_ranked(d, rank) == orc.index_bits(m, n, r, c, k, tile_rank=rank)
        Ip = (rng.random((T, r, k)) < 0.5).astype(np.uint8)
        Iz = (rng.random((T, k, c)) < 0.5).astype(np.uint8)
        ip, iz = lrbi.pack_factors(d, Ip, Iz, tile_rank=rank)
        # expected: the same arrays with everything unused cleared, packed by numpy
        Ipc, Izc = Ip.copy(), Iz.copy()
        tile_cols = -(-n // c)
        for t in range(T):
            ti, tj = divmod(t, tile_cols)
            Ipc[t, :, rank[t]:] = 0
            Izc[t, rank[t]:, :] = 0
            Ipc[t, max(0, min(r, m - ti * r)):, :] = 0
            Izc[t, :, max(0, min(c, n - tj * c)):] = 0
        ref_p = np.packbits(Ipc.reshape(T * r, k), axis=1, bitorder="little")
        ref_z = np.packbits(Izc.reshape(T * k, c), axis=1, bitorder="little")
        ipb, izb = ip.view(np.uint8).reshape(T * r, -1), iz.view(np.uint8).reshape(T * k, -1)
        assert np.array_equal(ipb[:, :ref_p.shape[1]], ref_p) and not ipb[:, ref_p.shape[1]:].any()
        assert np.array_equal(izb[:, :ref_z.shape[1]], ref_z) and not izb[:, ref_z.shape[1]:].any()
    d = lrbi.Desc(8, 8, 4, 4, 3)
    with pytest.raises(lrbi.LrbiError) as e:
        lrbi.index_bits_ranked(d, np.array([1, 2, 3, 4], np.int32))
    assert e.value.status == -3
    with pytest.raises(lrbi.LrbiError) as e:
        lrbi.pack_factors(d, np.zeros((4, 4, 3), np.uint8), np.zeros((4, 3, 4), np.uint8), tile_rank=[0, -1, 0, 0])
    assert e.value.status == -3


@pytest.mark.parametrize("r,c,k", [(5, 5, 2), (100, 100, 4), (3, 70, 33), (2, 130, 64), (4, 9, 100)])
def test_pack_factors_against_numpy_packbits(r, c, k):
    rng = np.random.default_rng(r * 1000 + c)
    T = 6
    d = lrbi.Desc(2 * r, 3 * c, r, c, k)
    Ip = (rng.random((T, r, k)) < 0.4).astype(np.uint8)
    Iz = (rng.random((T, k, c)) < 0.4).astype(np.uint8)
    ip, iz = lrbi.pack_factors(d, Ip * 3, Iz * 255)  # any non-zero byte is a set bit
    ipb = ip.view(np.uint8).reshape(T * r, -1)
    izb = iz.view(np.uint8).reshape(T * k, -1)
    ref_p = np.packbits(Ip.reshape(T * r, k), axis=1, bitorder="little")
    ref_z = np.packbits(Iz.reshape(T * k, c), axis=1, bitorder="little")
    assert np.array_equal(ipb[:, :ref_p.shape[1]], ref_p) and not ipb[:, ref_p.shape[1]:].any()
    assert np.array_equal(izb[:, :ref_z.shape[1]], ref_z) and not izb[:, ref_z.shape[1]:].any()
    assert ipb.shape[1] == 4 * ((k + 31) // 32) and izb.shape[1] == 8 * ((c + 63) // 64)


def test_unpack_mask_against_numpy():
    rng = np.random.default_rng(0)
    d = lrbi.Desc(6, 77, 3, 7, 2)
    M = (rng.random((6, 77)) < 0.5).astype(np.uint8)
    packed = np.zeros((6, 16), np.uint8)
    packed[:, :10] = np.packbits(M, axis=1, bitorder="little")
    assert np.array_equal(lrbi.unpack_mask(d, packed), M)


def test_gpu_entry_points_reject_bad_arguments_before_any_launch():
    lib = lrbi.load_library()
    d = lrbi.Desc(8, 128, 4, 64, 2)
    f = lib.lrbi_decode_mask
    # host memory is fine here: validation fails first, nothing is launched
    buf = (ctypes.c_uint8 * 4096)()
    base = (ctypes.addressof(buf) + 63) // 64 * 64  # 64-byte aligned address inside the buffer
    p = ctypes.c_void_p(base)
    assert f(ctypes.byref(d), None, p, p, 16, None) == -1
    assert f(ctypes.byref(d), p, p, p, 8, None) == -5       # pitch < ceil(n/8) and not a multiple of 16
    assert f(ctypes.byref(d), p, p, p, 24, None) == -5      # not a multiple of 16
    assert f(ctypes.byref(d), p, p, ctypes.c_void_p(base + 8), 16, None) == -6
    assert f(ctypes.byref(d), ctypes.c_void_p(base + 2), p, p, 16, None) == -6
    g = lib.lrbi_masked_gemm
    args = lambda **kw: [ctypes.byref(kw.get("d", d)), kw.get("dt", lrbi.F16), kw.get("W", p), kw.get("ldw", 128), p, p,
                         kw.get("X", p), kw.get("ldx", 16), kw.get("N", 16), kw.get("Y", p), kw.get("ldy", 16), None, 0,
                         None]
    assert g(*args(W=None)) == -1
    assert g(*args(dt=7)) == -4
    assert g(*args(N=0)) == -2
    assert g(*args(ldw=127)) == -5
    assert g(*args(ldx=15)) == -5
    assert g(*args(ldy=8)) == -5
    assert g(*args(W=ctypes.c_void_p(base + 1))) == -6
    assert g(*args(d=lrbi.Desc(8, 128, 4, 64, 2, lrbi.FLAG_PATH_MFMA), dt=lrbi.F32)) == -4
    assert g(*args(d=lrbi.Desc(8, 128, 4, 64, 2, lrbi.FLAG_PATH_MFMA), ldw=132)) == -6  # forced MFMA needs 16-byte rows
    # a forced split without workspace is refused
    d2 = lrbi.Desc(8, 1024, 4, 64, 2, lrbi.FLAG_PATH_MFMA | lrbi.flag_splitk(2))
    assert g(*args(d=d2, ldw=1024)) == -8
    assert lrbi.masked_gemm_workspace_bytes(d2, lrbi.F16, 16) == 2 * 8 * 16 * 4
    assert lrbi.masked_gemm_workspace_bytes(lrbi.Desc(4096, 4096, 512, 512, 32), lrbi.BF16, 1024) == 0
    assert lrbi.masked_gemm_workspace_bytes(lrbi.Desc(4096, 4096, 512, 512, 32), lrbi.BF16, 1) == 0
    # the fused decode + product entry point: the checks of both
    h = lib.lrbi_decode_and_gemm
    hargs = lambda **kw: [ctypes.byref(d), kw.get("dt", lrbi.F16), kw.get("W", p), kw.get("ldw", 128), p, p, p,
                          kw.get("ldx", 16), kw.get("N", 16), p, kw.get("ldy", 16), kw.get("M", p), kw.get("pitch", 16),
                          None, 0, None]
    assert h(*hargs(W=None)) == -1
    assert h(*hargs(M=None)) == -1
    assert h(*hargs(dt=7)) == -4
    assert h(*hargs(N=0)) == -2
    assert h(*hargs(ldw=127)) == -5
    assert h(*hargs(pitch=8)) == -5
    assert h(*hargs(pitch=24)) == -5
    assert h(*hargs(M=ctypes.c_void_p(base + 8))) == -6
    assert h(*hargs(W=ctypes.c_void_p(base + 1))) == -6


def test_threshold_eval_rejects_bad_arguments_before_any_launch():
    lib = lrbi.load_library()
    d = lrbi.Desc(8, 128, 4, 64, 2)
    buf = (ctypes.c_uint8 * 4096)()
    base = (ctypes.addressof(buf) + 63) // 64 * 64
    p = ctypes.c_void_p(base)
    f = lib.lrbi_threshold_eval
    args = lambda **kw: [ctypes.byref(kw.get("d", d)), kw.get("dt", lrbi.F16), kw.get("W", p), kw.get("ldw", 128), 0.5,
                         kw.get("method", 1), kw.get("amp", 1.0), kw.get("Mp", p), p, p, p, kw.get("Ip", None),
                         kw.get("Iz", None), kw.get("kept", p), p, None, 0, None]
    assert f(*args(W=None)) == -1
    assert f(*args(Mp=None)) == -1
    assert f(*args(kept=None)) == -1
    assert f(*args(Ip=p)) == -1                       # packed factors: both or neither
    assert f(*args(dt=9)) == -4
    assert f(*args(ldw=100)) == -5
    assert f(*args(W=ctypes.c_void_p(base + 1))) == -6
    assert f(*args(kept=ctypes.c_void_p(base + 4))) == -6
    assert f(*args(Ip=p, Iz=ctypes.c_void_p(base + 4))) == -6
    # magnitude manipulation of the cost: methods 1 .. 3, a positive finite amplification for method 3
    assert f(*args(method=0)) == -2 and f(*args(method=4)) == -2
    assert f(*args(method=3, amp=0.0)) == -2 and f(*args(method=3, amp=float("inf"))) == -2
    assert f(*args(method=3, amp=float("nan"))) == -2
    # factor bits of one tile must fit in 64 KiB of on-chip memory
    big = lrbi.Desc(4096, 65536, 4096, 65536, 8)
    assert f(*args(d=big, ldw=65536)) == -2
    # workspace: none needed when the tiles alone fill the chip, 16 bytes per (tile, band) otherwise
    assert lrbi.threshold_eval_workspace_bytes(lrbi.Desc(4096, 9216, 256, 256, 16)) == 0
    assert lrbi.threshold_eval_workspace_bytes(lrbi.Desc(4096, 4096, 512, 512, 32)) == 64 * 8 * 16
    assert lrbi.threshold_eval_workspace_bytes(lrbi.Desc(8, 128, 4, 64, 2)) == 0   # 4-row tiles: one band


def test_search_thresholds_rejects_bad_arguments_before_any_launch():
    lib = lrbi.load_library()
    d = lrbi.Desc(8, 128, 4, 64, 2)
    buf = (ctypes.c_uint8 * 4096)()
    base = (ctypes.addressof(buf) + 63) // 64 * 64
    p = ctypes.c_void_p(base)
    sweep = (ctypes.c_double * 3)(0.2, 0.5, 0.8)
    f = lib.lrbi_search_thresholds
    big = 1 << 30
    args = lambda **kw: [ctypes.byref(kw.get("d", d)), kw.get("dt", lrbi.F16), kw.get("W", p), kw.get("ldw", 128), 0.5,
                         kw.get("method", 1), kw.get("amp", 1.0), kw.get("Mp", p), p, kw.get("S", 0.9),
                         kw.get("sweep", sweep), kw.get("n_sp", 3),
                         kw.get("steps", 4), kw.get("tol", 1), kw.get("Tp", p), p, kw.get("kept", p), p,
                         kw.get("Ip", None), kw.get("Iz", None), kw.get("ws", p), kw.get("wsb", big), None]
    assert f(*args(W=None)) == -1
    assert f(*args(Mp=None)) == -1
    assert f(*args(sweep=None)) == -1
    assert f(*args(Tp=None)) == -1
    assert f(*args(ws=None)) == -1
    assert f(*args(Ip=p)) == -1
    assert f(*args(dt=9)) == -4
    assert f(*args(ldw=100)) == -5
    assert f(*args(n_sp=0)) == -2
    assert f(*args(steps=0)) == -2
    assert f(*args(tol=-1)) == -2
    assert f(*args(method=5)) == -2 and f(*args(method=3, amp=-2.0)) == -2
    assert f(*args(S=0.0)) == -2
    assert f(*args(S=1.0)) == -2
    assert f(*args(S=float("nan"))) == -2
    assert f(*args(sweep=(ctypes.c_double * 3)(0.2, 1.5, 0.8))) == -2
    assert f(*args(kept=ctypes.c_void_p(base + 4))) == -6
    assert f(*args(ws=ctypes.c_void_p(base + 8))) == -6
    assert f(*args(wsb=lrbi.search_workspace_bytes(d) - 1)) == -8
    # workspace: both sorted factors, the search state and the evaluation's scratch
    d2 = lrbi.Desc(4096, 9216, 256, 256, 16)
    assert lrbi.search_workspace_bytes(d2) >= 2 * 576 * 4096 * 4 + 576 * (64 + 4 + 4 + 8 + 8)
    assert lrbi.search_workspace_bytes(d2) < 2 * 576 * 4096 * 4 + 576 * 256
    # factors of more than 16384 entries take 2^j slots per tile
    d3 = lrbi.Desc(576, 1024, 576, 512, 145)
    assert lrbi.search_workspace_bytes(d3) >= 2 * (131072 + 131072) * 4


def test_backward_entry_points_reject_bad_arguments_before_any_launch():
    lib = lrbi.load_library()
    d = lrbi.Desc(8, 128, 4, 64, 2)
    buf = (ctypes.c_uint8 * 4096)()
    base = (ctypes.addressof(buf) + 63) // 64 * 64
    p = ctypes.c_void_p(base)
    t = lib.lrbi_masked_gemm_t
    targs = lambda **kw: [ctypes.byref(kw.get("d", d)), kw.get("dt", lrbi.F16), kw.get("W", p), kw.get("ldw", 128), p, p,
                          kw.get("dY", p), kw.get("lddy", 16), kw.get("N", 16), kw.get("dX", p), kw.get("lddx", 16), None,
                          0, None]
    assert t(*targs(W=None)) == -1
    assert t(*targs(dX=None)) == -1
    assert t(*targs(dt=7)) == -4
    assert t(*targs(N=0)) == -2
    assert t(*targs(ldw=127)) == -5
    assert t(*targs(lddy=15)) == -5
    assert t(*targs(lddx=8)) == -5
    assert t(*targs(dY=ctypes.c_void_p(base + 1))) == -6
    g = lib.lrbi_masked_grad
    gargs = lambda **kw: [ctypes.byref(kw.get("d", d)), kw.get("dt", lrbi.F16), kw.get("dY", p), kw.get("lddy", 16),
                          kw.get("X", p), kw.get("ldx", 16), kw.get("N", 16), p, p, kw.get("dW", p), kw.get("lddw", 128),
                          None]
    assert g(*gargs(dY=None)) == -1
    assert g(*gargs(dW=None)) == -1
    assert g(*gargs(dt=7)) == -4
    assert g(*gargs(N=-3)) == -2
    assert g(*gargs(lddw=127)) == -5
    assert g(*gargs(ldx=15)) == -5
    assert g(*gargs(X=ctypes.c_void_p(base + 1))) == -6
    # workspace of the transposed product: slices over m x n x N fp32 (N rounded up to 4); none for fp32
    big = lrbi.Desc(4096, 9216, 256, 256, 16)
    nb = lrbi.masked_gemm_t_workspace_bytes(big, lrbi.F16, 128)
    assert nb > 0 and nb % (9216 * 128 * 4) == 0
    assert lrbi.masked_gemm_t_workspace_bytes(big, lrbi.F32, 128) == 0
    nb1 = lrbi.masked_gemm_t_workspace_bytes(big, lrbi.F16, 1)  # one column: the tile kernel, split over m as well
    assert nb1 > 0 and nb1 % (9216 * 4 * 4) == 0


def test_lstm_step_rejects_bad_arguments_before_any_launch():
    lib = lrbi.load_library()
    d = lrbi.Desc(8, 128, 4, 64, 2)
    buf = (ctypes.c_uint8 * 4096)()
    base = (ctypes.addressof(buf) + 63) // 64 * 64
    p = ctypes.c_void_p(base)
    f = lib.lrbi_lstm_step
    args = lambda **kw: [ctypes.byref(kw.get("d", d)), kw.get("dt", lrbi.F16), kw.get("W", p), kw.get("ldw", 128), p, p,
                         kw.get("XH", p), kw.get("ldxh", 16), kw.get("B", 16), kw.get("C", p), kw.get("ldc", 16),
                         kw.get("H1", p), kw.get("ldh1", 16), kw.get("H2", None), kw.get("ldh2", 0), kw.get("ws", p),
                         kw.get("wsb", 1 << 30), None]
    assert f(*args(W=None)) == -1
    assert f(*args(C=None)) == -1
    assert f(*args(H1=None)) == -1
    assert f(*args(ws=None)) == -1
    assert f(*args(dt=lrbi.F32)) == -4
    assert f(*args(B=0)) == -2
    assert f(*args(d=lrbi.Desc(6, 128, 3, 64, 2))) == -2          # m must be 4 H
    assert f(*args(ldw=120)) == -5
    assert f(*args(ldc=8)) == -5
    assert f(*args(H2=p, ldh2=8)) == -5
    assert f(*args(ldw=132)) == -6                                 # W rows must be 16-byte pieces
    assert f(*args(C=ctypes.c_void_p(base + 2))) == -6
    assert f(*args(wsb=16)) == -8
    # one fp32 plane of the whole gate matrix per slice
    nb = lrbi.lstm_step_workspace_bytes(lrbi.Desc(6000, 3000, 300, 300, 8), lrbi.F16, 20)
    assert nb > 0 and nb % (6000 * 20 * 4) == 0


def test_nmf_rejects_bad_arguments_before_any_launch():
    lib = lrbi.load_library()
    d = lrbi.Desc(8, 128, 4, 64, 2)
    buf = (ctypes.c_uint8 * 4096)()
    base = (ctypes.addressof(buf) + 63) // 64 * 64
    p = ctypes.c_void_p(base)
    f = lib.lrbi_nmf
    args = lambda **kw: [ctypes.byref(kw.get("d", d)), kw.get("dt", lrbi.F16), kw.get("W", p), kw.get("ldw", 128),
                         kw.get("method", 1), 0.5, 2.0, kw.get("Mp", p), p, kw.get("iters", 3), kw.get("eps", 1e-9),
                         kw.get("ws", p), kw.get("wsb", 1 << 30), None]
    assert f(*args(W=None)) == -1
    assert f(*args(Mp=None)) == -1
    assert f(*args(ws=None)) == -1
    assert f(*args(dt=9)) == -4
    assert f(*args(d=lrbi.Desc(8, 128, 4, 64, 257))) == -3          # ranks above LRBI_MAX_RANK
    assert f(*args(method=0)) == -2
    assert f(*args(method=4)) == -2
    assert f(*args(iters=-1)) == -2
    assert f(*args(eps=0.0)) == -2
    assert f(*args(ldw=100)) == -5
    assert f(*args(Mp=ctypes.c_void_p(base + 2))) == -6
    assert f(*args(wsb=8)) == -8
    # a second copy of both factors and a k x k matrix per tile
    assert lrbi.nmf_workspace_bytes(lrbi.Desc(4096, 9216, 256, 256, 16)) == 2 * 576 * 256 * 16 * 4 + 576 * 16 * 16 * 4
