"""GPU parity for the generality of the format (Sec. 3.1): tiles cut off at the matrix edge and
tiles of different ranks, through every entry point, against the oracle."""
import numpy as np
import pytest
import torch

import paper_1905_05686_amd as lrbi
import workloads
from oracle import alg1
from oracle import lrbi_oracle as orc
from gpu_util import ORACLE_THREADS, TOL, desc_of, dev, to_device, to_float64, unpack_device_mask, workspace_for

pytestmark = pytest.mark.gpu

DT_CODE = {"f32": lrbi.F32, "f16": lrbi.F16, "bf16": lrbi.BF16}


def _cfg(m, n, r, c, k, p, N, dtype, seed=0):
    return workloads.Config("t", m, n, r, c, k, p, N, dtype, 0.05, seed)


def _device_factors(cfg, Ip01, Iz01, junk, tile_rank=None):
    """Packed factors on the device.  junk=True keeps whatever the 0/1 arrays hold in the positions a cut-off
    tile does not use (packed under a descriptor padded to whole tiles): the kernels must ignore them."""
    d = desc_of(cfg)
    if junk:
        assert tile_rank is None
        mp, np_ = -(-cfg.m // cfg.r) * cfg.r, -(-cfg.n // cfg.c) * cfg.c
        ip, iz = lrbi.pack_factors(lrbi.Desc(mp, np_, cfg.r, cfg.c, cfg.k), Ip01, Iz01)
    else:
        ip, iz = lrbi.pack_factors(d, Ip01, Iz01, tile_rank=tile_rank)
    return torch.from_numpy(ip.view(np.int32)).to(dev()), torch.from_numpy(iz.view(np.int64)).to(dev())


RAGGED = [
    # m, n, r, c, k, p
    (7, 9, 3, 4, 2, 0.4),
    (70, 90, 32, 40, 5, 0.3),
    (100, 129, 64, 64, 9, 0.2),          # one column beyond a tile
    (130, 1000, 128, 256, 16, 0.1),      # tile shapes the tuned kernels serve when they divide
    (577, 1000, 576, 512, 145, 0.02),    # the paper's tile shape, one row and a part of a tile beyond
    (33, 4000, 32, 4097, 3, 0.3),        # a single, cut-off tile column
    (255, 520, 256, 512, 40, 0.05),      # a single, cut-off tile row
]


@pytest.mark.parametrize("idx", range(len(RAGGED)))
@pytest.mark.parametrize("junk", [False, True])
def test_decode_edge_tiles(idx, junk):
    m, n, r, c, k, p = RAGGED[idx]
    cfg = _cfg(m, n, r, c, k, p, 1, "f32", seed=idx)
    print("decode edge tiles", RAGGED[idx], "junk", junk, flush=True)
    rng = np.random.default_rng(idx)
    Ip01, Iz01 = workloads.make_factors(rng, cfg.tiles, r, c, k, p)
    dIp, dIz = _device_factors(cfg, Ip01, Iz01, junk)
    pitch = ((n + 127) // 128) * 16 + 16
    out = torch.full((m, pitch), 0xEE, dtype=torch.uint8, device=dev())
    lrbi.decode_mask(desc_of(cfg), dIp, dIz, out=out)
    torch.cuda.synchronize()
    bits = unpack_device_mask(out, n)
    written = ((n + 127) // 128) * 128
    assert np.array_equal(bits[:, :n], orc.decode_mask(Ip01, Iz01, m, n, r, c, k))
    assert not bits[:, n:written].any(), "pad bits must be zero"
    assert (out.cpu().numpy()[:, written // 8:] == 0xEE).all()


RANKED = [
    # m, n, r, c, k, p, decode flags
    (512, 1024, 256, 256, 16, 0.1, 0),
    (512, 1024, 256, 256, 16, 0.1, lrbi.FLAG_DECODE_GENERIC),
    (192, 400, 64, 100, 40, 0.08, 0),
    (1152, 1024, 576, 512, 256, 0.015, 0),   # ranks drawn up to 256 on the paper's tile shape
    (130, 1000, 128, 256, 16, 0.1, 0),       # ranks and edge tiles together
]


@pytest.mark.parametrize("idx", range(len(RANKED)))
def test_decode_per_tile_rank(idx):
    m, n, r, c, k, p, flags = RANKED[idx]
    cfg = _cfg(m, n, r, c, k, p, 1, "f32", seed=20 + idx)
    print("decode per-tile rank", RANKED[idx], flush=True)
    rng = np.random.default_rng(20 + idx)
    Ip01, Iz01 = workloads.make_factors(rng, cfg.tiles, r, c, k, p)
    rank = rng.integers(0, k + 1, size=cfg.tiles).astype(np.int32)
    rank[0], rank[-1] = k, 0
    dIp, dIz = _device_factors(cfg, Ip01, Iz01, False, tile_rank=rank)
    out = lrbi.decode_mask(desc_of(cfg, flags), dIp, dIz)
    torch.cuda.synchronize()
    ref = orc.decode_mask(Ip01, Iz01, m, n, r, c, k, tile_rank=rank)
    assert np.array_equal(unpack_device_mask(out, n)[:, :n], ref)
    assert lrbi.index_bits_ranked(desc_of(cfg), rank) == orc.index_bits(m, n, r, c, k, tile_rank=rank)


GEMM = [
    # cfg, forced flags, junk, ranked
    (_cfg(70, 90, 32, 40, 5, 0.3, 1, "f32"), 0, True, False),
    (_cfg(70, 90, 32, 40, 5, 0.3, 3, "f32"), 0, False, True),
    (_cfg(130, 1000, 128, 256, 16, 0.1, 1, "bf16"), 0, True, False),          # matrix-vector, edge tiles
    (_cfg(130, 1000, 128, 256, 16, 0.1, 48, "f16"), 0, True, False),          # matrix cores, edge tiles
    (_cfg(577, 1000, 576, 512, 145, 0.02, 130, "bf16"), 0, True, False),
    (_cfg(255, 520, 256, 512, 40, 0.05, 16, "f16"), lrbi.FLAG_PATH_MFMA, True, False),
    (_cfg(300, 1096, 128, 256, 8, 0.15, 64, "bf16"), lrbi.FLAG_PATH_MFMA | lrbi.flag_splitk(3), False, True),
    (_cfg(512, 2048, 128, 256, 16, 0.1, 128, "bf16"), 0, False, True),        # dividing tiles, ranks: tuned kernel
    (_cfg(512, 2048, 128, 256, 16, 0.1, 1, "f16"), 0, False, True),
]


@pytest.mark.parametrize("idx", range(len(GEMM)))
def test_masked_gemm_edge_tiles_and_ranks(idx):
    cfg, flags, junk, ranked = GEMM[idx]
    print("gemm general", cfg, hex(flags), junk, ranked, flush=True)
    data = workloads.make(cfg)
    rank = None
    if ranked:
        rank = np.random.default_rng(idx).integers(0, cfg.k + 1, size=cfg.tiles).astype(np.int32)
        rank[0] = cfg.k
    dIp, dIz = _device_factors(cfg, data["Ip01"], data["Iz01"], junk, tile_rank=rank)
    desc = desc_of(cfg, flags)
    W, X = to_device(data["W"], cfg.dtype), to_device(data["X"], cfg.dtype)
    Y = lrbi.masked_gemm(desc, W, dIp, dIz, X, workspace=workspace_for(desc, DT_CODE[cfg.dtype], cfg.N))
    torch.cuda.synchronize()
    M = orc.decode_mask(data["Ip01"], data["Iz01"], cfg.m, cfg.n, cfg.r, cfg.c, cfg.k, tile_rank=rank)
    ref = orc.masked_gemm(workloads.to_float64(data["W"], cfg.dtype), M, workloads.to_float64(data["X"], cfg.dtype),
                          threads=ORACLE_THREADS)
    err = orc.rel_err(to_float64(Y), ref)
    print("rel_err %.3e" % err, flush=True)
    assert err <= TOL[cfg.dtype]


EVAL = [
    _cfg(7, 9, 3, 4, 2, 0.4, 1, "f32"),
    _cfg(70, 90, 32, 40, 5, 0.3, 1, "f16"),
    _cfg(130, 1000, 128, 256, 16, 0.1, 1, "bf16"),
    _cfg(1030, 520, 512, 512, 32, 0.06, 1, "bf16"),     # row bands, a last tile row of 6 rows
    _cfg(577, 1000, 576, 512, 145, 0.02, 1, "f16"),
]


@pytest.mark.parametrize("idx", range(len(EVAL)))
def test_threshold_eval_edge_tiles(idx):
    cfg = EVAL[idx]
    print("eval edge tiles", cfg, flush=True)
    data = workloads.make(cfg, want_x=False)
    f = workloads.make_real_factors(cfg)
    W64 = workloads.to_float64(data["W"], cfg.dtype)
    d = desc_of(cfg)
    t = lambda a: torch.from_numpy(a).to(dev())
    nbytes = lrbi.threshold_eval_workspace_bytes(d)
    ws = torch.empty(max(1, nbytes // 8), dtype=torch.int64, device=dev()) if nbytes else None
    kept, cost, ip, iz = lrbi.threshold_eval(d, to_device(data["W"], cfg.dtype), f["w_threshold"], t(f["Mp"]), t(f["Mz"]),
                                             t(f["Tp"]), t(f["Tz"]), want_factors=True, workspace=ws)
    torch.cuda.synchronize()
    Ip, Iz = orc.threshold_factors(f["Mp"], f["Mz"], f["Tp"], f["Tz"])
    M = orc.decode_mask(Ip, Iz, cfg.m, cfg.n, cfg.r, cfg.c, cfg.k)
    kept_ref, cost_ref = orc.candidate_cost(W64, f["w_threshold"], M, cfg.r, cfg.c)
    assert np.array_equal(kept.cpu().numpy().astype(np.uint64), kept_ref)
    assert np.all(np.abs(cost.cpu().numpy() - cost_ref) <= 1e-12 * np.maximum(cost_ref, 1.0))
    # packed factors: what a cut-off tile does not use is written as zero, as the host packer writes it
    ip_ref, iz_ref = lrbi.pack_factors(d, Ip, Iz)
    assert np.array_equal(ip.cpu().numpy().view(np.uint32).reshape(-1), np.asarray(ip_ref).view(np.uint32).reshape(-1))
    assert np.array_equal(iz.cpu().numpy().view(np.uint32).reshape(-1), np.asarray(iz_ref).view(np.uint32).reshape(-1))


SEARCH = [
    (_cfg(7, 9, 3, 4, 2, 0.4, 1, "f32"), 0.6, 5, 1),
    (_cfg(70, 90, 32, 40, 5, 0.3, 1, "f16"), 0.85, 7, 6),
    (_cfg(130, 1000, 128, 256, 16, 0.1, 1, "bf16"), 0.9, 8, 40),
    (_cfg(577, 600, 576, 512, 40, 0.02, 1, "f16"), 0.8, 4, 500),   # 23040-entry factors: sorted in the workspace
]


@pytest.mark.parametrize("idx", range(len(SEARCH)))
def test_search_edge_tiles(idx):
    cfg, S, steps, tol = SEARCH[idx]
    print("search edge tiles", cfg, flush=True)
    sweep = [0.2, 0.5, 0.8, 0.95]
    data = workloads.make(cfg, want_x=False)
    f = workloads.make_real_factors(cfg)
    W64 = workloads.to_float64(data["W"], cfg.dtype)
    t = lambda a: torch.from_numpy(a).to(dev())
    Tp, Tz, kept, cost, ip, iz = lrbi.search_thresholds(desc_of(cfg), to_device(data["W"], cfg.dtype), f["w_threshold"],
                                                        t(f["Mp"]), t(f["Mz"]), S, sweep, steps, tol, want_factors=True)
    torch.cuda.synchronize()
    rtp, rtz, rk, rc = alg1.search_thresholds(W64, f["w_threshold"], f["Mp"], f["Mz"], cfg.r, cfg.c, S, sweep, steps, tol)
    Tp, Tz = Tp.cpu().numpy(), Tz.cpu().numpy()
    cost = cost.cpu().numpy()
    assert np.all(np.abs(cost - rc) <= 1e-12 * np.maximum(rc, 1.0))
    same = (Tp == rtp) & (Tz == rtz)
    assert same.mean() >= 0.9 and np.array_equal(kept.cpu().numpy().astype(np.uint64)[same], rk[same])
    Ip, Iz = orc.threshold_factors(f["Mp"], f["Mz"], Tp, Tz)
    ip_ref, iz_ref = lrbi.pack_factors(desc_of(cfg), Ip, Iz)
    assert np.array_equal(ip.cpu().numpy().view(np.uint32).reshape(-1), np.asarray(ip_ref).view(np.uint32).reshape(-1))
    assert np.array_equal(iz.cpu().numpy().view(np.uint32).reshape(-1), np.asarray(iz_ref).view(np.uint32).reshape(-1))
