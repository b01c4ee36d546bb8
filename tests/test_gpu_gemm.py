"""GPU parity: lrbi_masked_gemm against the fp64 CPU oracle."""
import numpy as np
import pytest
import torch

import paper_1905_05686_amd as lrbi
import workloads
from oracle import lrbi_oracle as orc
from gpu_util import (ORACLE_THREADS, TOL, TORCH_DTYPE, desc_of, dev, device_factors, to_device, to_float64,
                      unpack_device_mask, workspace_for)

pytestmark = pytest.mark.gpu

DT_CODE = {"f32": lrbi.F32, "f16": lrbi.F16, "bf16": lrbi.BF16}


def _run(cfg, data, flags=0, use_workspace=True, ldpad=0):
    desc = desc_of(cfg, flags)
    dIp, dIz = device_factors(desc, data["Ip01"], data["Iz01"])
    W = to_device(data["W"], cfg.dtype)
    X = to_device(data["X"], cfg.dtype)
    if ldpad:
        Wp = torch.zeros((cfg.m, cfg.n + ldpad), dtype=W.dtype, device=dev())
        Wp[:, :cfg.n] = W
        W = Wp[:, :cfg.n]
        Xp = torch.zeros((cfg.n, cfg.N + ldpad), dtype=X.dtype, device=dev())
        Xp[:, :cfg.N] = X
        X = Xp[:, :cfg.N]
    ws = workspace_for(desc, DT_CODE[cfg.dtype], cfg.N) if use_workspace else None
    Y = lrbi.masked_gemm(desc, W, dIp, dIz, X, workspace=ws)
    torch.cuda.synchronize()
    return Y


def _oracle(cfg, data):
    M = orc.decode_mask(data["Ip01"], data["Iz01"], cfg.m, cfg.n, cfg.r, cfg.c, cfg.k)
    return orc.masked_gemm(workloads.to_float64(data["W"], cfg.dtype), M, workloads.to_float64(data["X"], cfg.dtype),
                           threads=ORACLE_THREADS), M


def _assert_close(Y, ref, dtype, what=""):
    err = orc.rel_err(to_float64(Y), ref)
    normwise = float(np.max(np.abs(to_float64(Y) - ref)) / max(np.max(np.abs(ref)), 1e-300))
    print("%s rel_err %.3e (normwise %.3e, tol %.0e)" % (what, err, normwise, TOL[dtype]), flush=True)
    assert err <= TOL[dtype], (what, err)


@pytest.mark.parametrize("name", ["C1", "C2", "C3a", "C3b", "C4", "C5"])
def test_config_parity(name):
    cfg = workloads.CONFIGS[name]
    print("gemm config", name, flush=True)
    data = workloads.make(cfg)
    ref, _ = _oracle(cfg, data)
    Y = _run(cfg, data)
    _assert_close(Y, ref, cfg.dtype, name)
    # run-to-run identical bits (no floating-point atomics anywhere)
    Y2 = _run(cfg, data)
    assert torch.equal(Y.view(torch.int16 if Y.element_size() == 2 else torch.int32),
                       Y2.view(torch.int16 if Y.element_size() == 2 else torch.int32))


def _small(m, n, r, c, k, p, N, dtype, seed=0, sigma=0.05):
    return workloads.Config("t", m, n, r, c, k, p, N, dtype, sigma, seed)


EDGE = [
    # shape                                         forced flags
    (_small(96, 200, 48, 100, 4, 0.2, 1, "f32"), 0),
    (_small(96, 200, 48, 100, 4, 0.2, 7, "f32"), 0),
    (_small(33, 77, 3, 7, 3, 0.3, 2, "f32"), 0),             # nothing aligned: scalar loads everywhere
    (_small(130, 4104, 65, 1368, 9, 0.1, 1, "bf16"), lrbi.FLAG_PATH_VALU),  # n spans three 2048-column segments
    (_small(130, 4104, 65, 1368, 9, 0.1, 3, "f16"), 0),
    (_small(128, 192, 64, 64, 8, 0.2, 128, "bf16"), 0),      # one 128x128 tile, 3 slabs
    (_small(300, 2400, 300, 300, 8, 0.12, 20, "f16"), lrbi.FLAG_PATH_MFMA),  # unaligned tiles, scalar X path, split
    (_small(3000, 600, 300, 300, 8, 0.12, 20, "f16"), 0),    # the row-streaming kernel by itself: 190 workgroups, the last of a tile row with 12 rows
    (_small(2100, 512, 300, 128, 6, 0.15, 8, "bf16"), 0),    # the same, bf16, 7 tile rows of 19 workgroups
    (_small(384, 1024, 128, 256, 16, 0.1, 72, "f16"), 0),    # 128x64 tile variant (N in 33..64 -> padded)
    (_small(384, 1024, 128, 256, 16, 0.1, 40, "bf16"), 0),
    (_small(384, 1024, 128, 256, 16, 0.1, 48, "bf16"), lrbi.FLAG_PATH_MFMA | lrbi.flag_tile(10)),  # the 128 x 64 panel kernel by flag
    (_small(384, 1024, 128, 256, 16, 0.1, 44, "f16"), 0),    # N no multiple of 8: the 128 x 64 panel kernel by itself
    (_small(200, 1000, 100, 500, 40, 0.05, 136, "bf16"), 0), # rank above 32, ragged m and N
    (_small(256, 2048, 128, 512, 32, 0.06, 256, "bf16"), lrbi.FLAG_PATH_MFMA | lrbi.flag_splitk(4)),
    (_small(256, 2048, 128, 512, 32, 0.06, 256, "f16"), lrbi.FLAG_PATH_MFMA | lrbi.flag_splitk(1)),
    (_small(256, 512, 128, 128, 8, 0.2, 2, "f16"), lrbi.FLAG_PATH_MFMA),   # tiny batch forced onto MFMA
    (_small(256, 512, 128, 128, 8, 0.2, 64, "bf16"), lrbi.FLAG_PATH_VALU), # big batch forced onto the ALUs
    (_small(256, 512, 128, 128, 8, 0.2, 96, "bf16"), lrbi.FLAG_PATH_MFMA | lrbi.flag_tile(2)),
    (_small(256, 512, 128, 128, 8, 0.2, 96, "bf16"), lrbi.FLAG_PATH_MFMA | lrbi.flag_tile(3)),
    # tile shape and ranks of the paper's own experiments (Sec. 4: 576 x 512 tiles, rank 145; Table 1: rank 256)
    (_small(1152, 1024, 576, 512, 145, 0.02, 64, "f16"), 0),
    (_small(1152, 1024, 576, 512, 256, 0.015, 1, "bf16"), 0),
    (_small(64, 576, 64, 576, 8, 0.2, 12416, "bf16"), 0),    # few rows, many columns: 64-column blocks, unsplit
    (_small(48, 288, 16, 96, 4, 0.3, 3080, "f16"), 0),       # ... 32-column blocks
    (_small(4096, 2304, 256, 256, 16, 0.08, 3, "bf16"), 0),  # three columns of a large matrix: the tile kernel, mostly idle
    # few rows, short rows: the row-streaming kernels on a grid far smaller than the chip (automatic choice)
    (_small(1200, 600, 1200, 600, 145, 0.05, 20, "f16"), 0), # the gate matrix of an LSTM layer of size 300 (Sec. 4), untiled, at Table 2's rank 145
    (_small(800, 400, 800, 400, 145, 0.05, 20, "f16"), 0),   # 50 workgroups
    (_small(128, 1024, 128, 256, 16, 0.1, 8, "f16"), 0),     # eight workgroups
    (_small(64, 4096, 64, 256, 16, 0.1, 1, "bf16"), 0),      # eight workgroups of the single-column kernel
    # tile widths that are an odd multiple of 64 on the pipelined tile kernel (Table 2's 576-column tiles): 128-column
    # units of the mask that lie across two tile columns
    (_small(256, 1152, 128, 576, 8, 0.2, 128, "f16"), 0),      # two tile columns, three panels, the last one short
    (_small(256, 3456, 128, 576, 40, 0.05, 136, "bf16"), 0),   # two I_p words per row, two column blocks, ragged N
    (_small(128, 9216, 128, 576, 32, 0.054, 128, "f16"), 0),   # split over n: slices begin inside tiles
    (_small(256, 768, 256, 192, 16, 0.1, 72, "bf16"), 0),      # 192-column tiles
    (_small(128, 512, 128, 64, 8, 0.2, 128, "f16"), 0),        # 64-column tiles: every unit has two tiles
    (_small(256, 1152, 128, 576, 8, 0.2, 64, "f16"), 0),       # 33 to 64 columns on these widths: the same kernel, half a block
    (_small(256, 1152, 128, 576, 8, 0.2, 40, "bf16"), 0),
    (_small(256, 2304, 128, 576, 16, 0.1, 256, "bf16"), lrbi.FLAG_PATH_MFMA | lrbi.flag_splitk(3)),
]


@pytest.mark.parametrize("idx", range(len(EDGE)))
def test_edge_shapes(idx):
    cfg, flags = EDGE[idx]
    print("gemm edge", idx, cfg, hex(flags), flush=True)
    data = workloads.make(cfg)
    ref, _ = _oracle(cfg, data)
    _assert_close(_run(cfg, data, flags=flags), ref, cfg.dtype, "edge%d" % idx)


# The row-streaming kernel (narrow batches), forced so that small matrices take it too; the configurations C3a and
# C4 above reach it on their own.
STREAM = [
    _small(100, 200, 50, 100, 4, 0.2, 1, "bf16"),        # last workgroup has 4 of its 16 rows, one short slab
    _small(130, 4104, 65, 1368, 9, 0.1, 4, "f16"),       # 16 slabs and 8 columns; tiles cut through slabs and words
    _small(300, 2400, 300, 300, 8, 0.12, 20, "f16"),     # C4's tiles and batch
    _small(256, 512, 128, 128, 8, 0.2, 32, "bf16"),      # both 16-column blocks full
    _small(48, 264, 24, 33, 5, 0.3, 8, "f16"),           # tiles narrower than two mask words
    _small(1152, 1024, 576, 512, 145, 0.02, 16, "f16"),  # rank 145: five I_p words per row
    _small(64, 520, 32, 130, 6, 0.25, 12, "bf16"),
    _small(64, 520, 32, 130, 6, 0.25, 28, "f16"),
    _small(2048, 8, 512, 8, 2, 0.5, 1, "f16"),           # a single 16-byte piece per row
    _small(64, 96, 32, 32, 3, 0.3, 8, "bf16"),           # a tile row's I_z is no whole number of 16-byte pieces
    # one column: a row travels in registers (rows of up to 8192 columns; 2, 4, 8 or 16 pieces of 1 KB)
    _small(130, 4104, 65, 1368, 9, 0.1, 1, "bf16"),      # 16 pieces, the ninth holds 8 columns; tiles cut through words
    _small(64, 4096, 32, 512, 32, 0.1, 1, "f16"),        # 8 full pieces
    _small(72, 8192, 24, 1024, 16, 0.08, 1, "bf16"),     # 16 full pieces
    _small(1152, 1024, 576, 512, 145, 0.02, 1, "f16"),   # 2 pieces, rank 145
    _small(44, 1544, 22, 772, 7, 0.2, 1, "f16"),         # 4 pieces, the last one short; 6 of 8 rows in the last workgroup
    _small(40, 8704, 20, 1088, 6, 0.15, 1, "bf16"),      # longer rows: back on the staged kernel, 17 slabs of 512
]


@pytest.mark.parametrize("idx", range(len(STREAM)))
def test_row_streaming_kernel(idx):
    cfg = STREAM[idx]
    print("gemm stream", idx, cfg, flush=True)
    data = workloads.make(cfg)
    ref, M = _oracle(cfg, data)
    Y = _run(cfg, data, flags=lrbi.FLAG_PATH_STREAM)
    _assert_close(Y, ref, cfg.dtype, "stream%d" % idx)
    # nothing stored under a pruned bit reaches Y, also not through the clamped loads past the last row and column
    W = workloads.to_float64(data["W"], cfg.dtype).astype(np.float32)
    poison = np.where(np.arange(cfg.n)[None, :] % 2 == 0, np.nan, np.inf).astype(np.float32)
    data["W"] = workloads.to_storage(np.where(M == 1, W, poison), cfg.dtype)
    Yp = _run(cfg, data, flags=lrbi.FLAG_PATH_STREAM)
    assert torch.equal(Y.view(torch.int16), Yp.view(torch.int16))


def test_row_streaming_kernel_refuses_what_it_cannot_serve():
    cfg = _small(64, 520, 32, 130, 6, 0.25, 6, "f16")  # N = 6: neither 1 nor a multiple of 4
    data = workloads.make(cfg)
    with pytest.raises(lrbi.LrbiError):
        _run(cfg, data, flags=lrbi.FLAG_PATH_STREAM)
    cfg = _small(64, 520, 32, 130, 6, 0.25, 1, "f32")
    with pytest.raises(lrbi.LrbiError):
        _run(cfg, workloads.make(cfg), flags=lrbi.FLAG_PATH_STREAM)


@pytest.mark.parametrize("dtype,N", [("bf16", 1), ("f16", 20)])
def test_row_streaming_identity_x_returns_masked_weights_exactly(dtype, N):
    cfg = _small(256, 256, 128, 128, 8, 0.2, N, dtype)
    data = workloads.make(cfg)
    X = np.zeros((cfg.n, N), np.float32)
    X[np.arange(N), np.arange(N)] = 1.0
    data["X"] = workloads.to_storage(X, dtype)
    M = orc.decode_mask(data["Ip01"], data["Iz01"], cfg.m, cfg.n, cfg.r, cfg.c, cfg.k)
    Wm = np.where(M == 1, workloads.to_float64(data["W"], dtype), 0.0)
    Y = to_float64(_run(cfg, data, flags=lrbi.FLAG_PATH_STREAM))
    assert np.array_equal(Y, Wm[:, :N])


def test_padded_leading_dimensions():
    for cfg in (_small(128, 256, 64, 128, 8, 0.2, 24, "f16"), _small(128, 256, 64, 128, 8, 0.2, 1, "bf16"),
                _small(50, 120, 25, 60, 4, 0.2, 3, "f32")):
        for pad in (8, 3):
            print("gemm ldpad", cfg.dtype, cfg.N, pad, flush=True)
            data = workloads.make(cfg)
            ref, _ = _oracle(cfg, data)
            _assert_close(_run(cfg, data, ldpad=pad), ref, cfg.dtype, "ldpad")


def test_without_workspace_falls_back_to_unsplit_kernel():
    cfg = _small(300, 2400, 300, 300, 8, 0.12, 20, "f16")
    data = workloads.make(cfg)
    assert lrbi.masked_gemm_workspace_bytes(desc_of(cfg), lrbi.F16, cfg.N) > 0
    ref, _ = _oracle(cfg, data)
    _assert_close(_run(cfg, data, flags=lrbi.FLAG_PATH_MFMA, use_workspace=False), ref, cfg.dtype, "no-ws")
    with pytest.raises(lrbi.LrbiError) as e:
        _run(cfg, data, flags=lrbi.FLAG_PATH_MFMA | lrbi.flag_splitk(2), use_workspace=False)
    assert e.value.status == -8


@pytest.mark.parametrize("dtype,N", [("f16", 256), ("bf16", 256), ("bf16", 1), ("f32", 1), ("f16", 20)])
def test_identity_x_returns_masked_weights_exactly(dtype, N):
    # X = [I | 0]: Y[:, q] = (W o M)[:, q] bit for bit, which isolates the masking
    cfg = _small(256, 256, 128, 128, 8, 0.2, N, dtype)
    data = workloads.make(cfg)
    X = np.zeros((cfg.n, N), np.float32)
    X[np.arange(min(N, cfg.n)), np.arange(min(N, cfg.n))] = 1.0
    data["X"] = workloads.to_storage(X, dtype)
    M = orc.decode_mask(data["Ip01"], data["Iz01"], cfg.m, cfg.n, cfg.r, cfg.c, cfg.k)
    Wm = np.where(M == 1, workloads.to_float64(data["W"], dtype), 0.0)
    Y = to_float64(_run(cfg, data))
    assert np.array_equal(Y, Wm[:, :N])


@pytest.mark.parametrize("dtype,N", [("f16", 128), ("bf16", 128), ("bf16", 1), ("f32", 2)])
def test_values_under_pruned_bits_never_reach_y(dtype, N):
    cfg = _small(256, 512, 128, 256, 8, 0.15, N, dtype)
    data = workloads.make(cfg)
    ref, M = _oracle(cfg, data)
    W = workloads.to_float64(data["W"], dtype).astype(np.float32)
    poison = np.where(np.arange(cfg.n)[None, :] % 2 == 0, np.nan, np.inf).astype(np.float32)
    W = np.where(M == 1, W, poison)
    data["W"] = workloads.to_storage(W, dtype)
    Y = _run(cfg, data)
    assert torch.isfinite(Y).all()
    _assert_close(Y, ref, dtype, "poison")


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_output_rounding_is_nearest_even(dtype):
    # small integers: every product and partial sum is exact in fp32, so the only rounding
    # is the final one, which must be round-to-nearest-even of the exact result
    cfg = _small(128, 512, 128, 256, 8, 0.3, 128, dtype)
    rng = np.random.default_rng(5)
    data = workloads.make(cfg)
    data["W"] = workloads.to_storage(rng.integers(-8, 9, (cfg.m, cfg.n)).astype(np.float32), dtype)
    data["X"] = workloads.to_storage(rng.integers(-8, 9, (cfg.n, cfg.N)).astype(np.float32), dtype)
    ref, _ = _oracle(cfg, data)
    assert np.abs(ref).max() > 256  # beyond bf16's exact-integer range, so rounding really happens
    exp = workloads.to_float64(workloads.to_storage(ref, dtype), dtype)
    Y = to_float64(_run(cfg, data))
    assert np.array_equal(Y, exp)


def test_all_ones_factors_equal_dense_product():
    cfg = _small(256, 512, 128, 128, 4, 1.0, 128, "bf16")
    data = workloads.make(cfg)
    assert data["Ip01"].all() and data["Iz01"].all()
    Y = _run(cfg, data)
    ref = workloads.to_float64(data["W"], "bf16") @ workloads.to_float64(data["X"], "bf16")
    _assert_close(Y, ref, "bf16", "dense")
    zero = dict(data, Ip01=data["Ip01"] * 0)
    assert not to_float64(_run(cfg, zero)).any()


def test_full_size_sampled_rows_in_bench_configuration():
    """C2 at full size in the launch configuration bench.py times, checked on rows the
    oracle computes one by one (independent of test_config_parity's whole-matrix check)."""
    cfg = workloads.CONFIGS["C2"]
    data = workloads.make(cfg)
    Y = to_float64(_run(cfg, data))
    Wd = workloads.to_float64(data["W"], cfg.dtype)
    Xd = workloads.to_float64(data["X"], cfg.dtype)
    tile_cols = cfg.n // cfg.c
    rng = np.random.default_rng(3)
    rms = float(np.sqrt(np.mean(Y * Y)))
    for i in [0, cfg.m - 1] + [int(v) for v in rng.integers(cfg.m, size=30)]:
        ti, il = divmod(i, cfg.r)
        row = np.zeros(cfg.N)
        for tj in range(tile_cols):
            t = ti * tile_cols + tj
            bits = orc.decode_mask(data["Ip01"][t:t + 1, il:il + 1], data["Iz01"][t:t + 1], 1, cfg.c, 1, cfg.c, cfg.k)
            row += orc.masked_gemm(Wd[i:i + 1, tj * cfg.c:(tj + 1) * cfg.c], bits, Xd[tj * cfg.c:(tj + 1) * cfg.c])[0]
        err = np.max(np.abs(Y[i] - row) / np.maximum(np.abs(row), rms))
        assert err <= TOL[cfg.dtype], (i, err)


# ---- mask and product from one call (rows a1-a6 fused)
FUSED = [
    _small(256, 1152, 128, 128, 8, 0.2, 128, "f16"),     # the tile kernel leaves the mask: one column block, unsplit
    _small(256, 1024, 256, 256, 16, 0.1, 256, "bf16"),   # two column blocks: only the first one stores the mask
    _small(256, 1024, 256, 256, 16, 0.1, 48, "bf16"),    # 33 to 64 columns: the same kernel, part of its column block idle
    _small(128, 9216, 128, 256, 16, 0.08, 128, "f16"),   # split over n: every slice stores its own units, last panel short
    (_small(300, 2400, 300, 300, 8, 0.12, 20, "f16"), lrbi.FLAG_PATH_MFMA),  # generic tile kernel, 32-column blocks, tiles cut through mask words
    _small(1200, 600, 1200, 600, 145, 0.05, 20, "f16"),  # few, short rows (an LSTM layer of size 300 at rank 145): the ring kernel on 75 workgroups
    _small(130, 264, 65, 33, 5, 0.3, 70, "bf16"),        # generic tile kernel, tiles narrower than two mask words
    _small(260, 520, 128, 128, 8, 0.2, 96, "f16"),       # generic kernel on cut-off aligned tiles: 8 bits of the last piece live
    _small(1152, 1024, 576, 512, 145, 0.02, 64, "f16"),  # rank 145
    _small(256, 1088, 128, 64, 8, 0.2, 200, "bf16"),     # two blocks of columns, n a multiple of 64 but not of 128
    _small(50, 120, 25, 60, 4, 0.2, 3, "f32"),
    workloads.CONFIGS["C2"],                             # the benchmark's workload at full size
    # the pipelined tile kernel on tile widths of 64 (2 j + 1): mask units gathered per 64-column half
    _small(256, 1152, 128, 576, 8, 0.2, 128, "f16"),
    _small(256, 3456, 128, 576, 40, 0.05, 136, "bf16"),
    _small(128, 9216, 128, 576, 32, 0.054, 128, "f16"),
    _small(128, 512, 128, 64, 8, 0.2, 128, "f16"),
    _small(256, 1152, 128, 576, 8, 0.2, 40, "bf16"),
    workloads.Config("paper_fc5_tiles", 4096, 9216, 512, 576, 32, 0.054, 128, "f16", 0.01),  # Table 2's tiling of C2's layer
    # narrow batches with enough rows for the row-streaming kernels: they store the rows' mask from LDS
    _small(3000, 600, 300, 300, 8, 0.12, 20, "f16"),     # ring kernel, tiles cut through mask words, last workgroups short
    _small(2048, 1024, 256, 128, 8, 0.15, 1, "bf16"),    # single-column kernel
    _small(1040, 4104, 65, 1368, 9, 0.1, 1, "bf16"),     # single-column kernel, n no multiple of 128: the last piece's pad bits
    _small(1040, 8704, 520, 1088, 6, 0.15, 1, "bf16"),   # one column over rows longer than 8192: the ring kernel's 8-row form
    workloads.CONFIGS["C3a"],
    workloads.CONFIGS["C4"],
]


@pytest.mark.parametrize("N", [1, 8, 128])
def test_fp16_subnormal_weights_are_not_flushed(N):
    """Weights below fp16's smallest normal number (2^-14) times inputs of 2^10: exact in fp32, and far above zero in
    the sum; a path that flushes subnormal operands (the 2-element dot products of the single-column kernel, the
    matrix cores of the others) would return zeros."""
    cfg = _small(128, 1024, 128, 256, 8, 0.3, N, "f16")
    rng = np.random.default_rng(11)
    data = workloads.make(cfg)
    data["W"] = (rng.integers(1, 64, (cfg.m, cfg.n)).astype(np.float32) * np.float32(2.0 ** -24)).astype(np.float16)
    data["X"] = np.full((cfg.n, cfg.N), 1024.0, dtype=np.float16)
    ref, M = _oracle(cfg, data)
    assert np.abs(ref).max() > 1e-3 and M.sum() > 0
    Y = to_float64(_run(cfg, data))
    # every product k * 2^-14 and every partial sum is exact in fp32; only the final rounding to fp16 is left
    exp = workloads.to_float64(workloads.to_storage(ref, "f16"), "f16")
    assert np.array_equal(Y, exp)


@pytest.mark.parametrize("idx", range(len(FUSED)))
def test_decode_and_gemm_equals_the_two_calls(idx):
    cfg, flags = FUSED[idx] if isinstance(FUSED[idx], tuple) else (FUSED[idx], 0)
    print("decode_and_gemm", idx, cfg, hex(flags), flush=True)
    data = workloads.make(cfg)
    desc = desc_of(cfg, flags)
    dIp, dIz = device_factors(desc, data["Ip01"], data["Iz01"])
    W, X = to_device(data["W"], cfg.dtype), to_device(data["X"], cfg.dtype)
    ws = workspace_for(desc, DT_CODE[cfg.dtype], cfg.N)
    pitch = ((cfg.n + 127) // 128) * 16 + 32
    mask = torch.full((cfg.m, pitch), 0xA5, dtype=torch.uint8, device=dev())
    mask2 = torch.full((cfg.m, pitch), 0xA5, dtype=torch.uint8, device=dev())
    m1, Y1 = lrbi.decode_and_gemm(desc, W, dIp, dIz, X, mask=mask, workspace=ws)
    lrbi.decode_mask(desc, dIp, dIz, out=mask2)
    Y2 = lrbi.masked_gemm(desc, W, dIp, dIz, X, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(m1, mask2)  # the bytes beyond the written part of a row are left alone by both
    assert torch.equal(Y1.view(torch.uint8), Y2.view(torch.uint8))
    # and against the oracle
    M = orc.decode_mask(data["Ip01"], data["Iz01"], cfg.m, cfg.n, cfg.r, cfg.c, cfg.k)
    assert np.array_equal(unpack_device_mask(m1, cfg.n)[:, :cfg.n], M)
    ref, _ = _oracle(cfg, data)
    _assert_close(Y1, ref, cfg.dtype, "fused%d" % idx)
