"""GPU parity of the backward pass through the masking layer (Sec. 2): lrbi_masked_gemm_t (dX = (W o I_a)^T dY) and
lrbi_masked_grad (dW = (dY X^T) o I_a) against the fp64 oracle."""
import numpy as np
import pytest
import torch

import paper_1905_05686_amd as lrbi
import workloads
from oracle import lrbi_oracle as orc
from gpu_util import TOL, desc_of, dev, device_factors, to_device, to_float64

pytestmark = pytest.mark.gpu

DT_CODE = {"f32": lrbi.F32, "f16": lrbi.F16, "bf16": lrbi.BF16}


def _inputs(cfg):
    data = workloads.make(cfg)
    rng = np.random.default_rng(cfg.seed + 77)
    dY = workloads.to_storage(rng.standard_normal((cfg.m, cfg.N), dtype=np.float32), cfg.dtype)
    return data, dY


def _padded(t, pad):
    if not pad:
        return t
    p = torch.zeros((t.shape[0], t.shape[1] + pad), dtype=t.dtype, device=t.device)
    p[:, :t.shape[1]] = t
    return p[:, :t.shape[1]]


def _check(cfg, ldpad=0, use_workspace=True, what=""):
    print("backward", what, cfg, "ldpad", ldpad, flush=True)
    data, dYs = _inputs(cfg)
    desc = desc_of(cfg)
    dIp, dIz = device_factors(desc, data["Ip01"], data["Iz01"])
    W = _padded(to_device(data["W"], cfg.dtype), ldpad)
    X = _padded(to_device(data["X"], cfg.dtype), ldpad)
    dY = _padded(to_device(dYs, cfg.dtype), ldpad)
    ws = None
    nbytes = lrbi.masked_gemm_t_workspace_bytes(desc, DT_CODE[cfg.dtype], cfg.N)
    if use_workspace and nbytes:
        ws = torch.empty(nbytes // 4, dtype=torch.float32, device=dev())
    dX = lrbi.masked_gemm_t(desc, W, dIp, dIz, dY, workspace=ws)
    dW = lrbi.masked_grad(desc, dY, X, dIp, dIz)
    torch.cuda.synchronize()
    M = orc.decode_mask(data["Ip01"], data["Iz01"], cfg.m, cfg.n, cfg.r, cfg.c, cfg.k)
    W64, X64, dY64 = (workloads.to_float64(a, cfg.dtype) for a in (data["W"], data["X"], dYs))
    e1 = orc.rel_err(to_float64(dX), orc.masked_gemm_t(W64, M, dY64))
    dW_ref = orc.masked_grad(dY64, X64, M)
    dWh = to_float64(dW)
    e2 = orc.rel_err(dWh, dW_ref)
    print("dX rel_err %.3e  dW rel_err %.3e (tol %.0e)" % (e1, e2, TOL[cfg.dtype]), flush=True)
    assert e1 <= TOL[cfg.dtype] and e2 <= TOL[cfg.dtype]
    assert not dWh[M == 0].any(), "pruned weights must get exactly zero"
    # identical bits from call to call
    dX2 = lrbi.masked_gemm_t(desc, W, dIp, dIz, dY, workspace=ws)
    dW2 = lrbi.masked_grad(desc, dY, X, dIp, dIz)
    view = torch.int16 if dX.element_size() == 2 else torch.int32
    assert torch.equal(dX.view(view), dX2.view(view)) and torch.equal(dW.view(view), dW2.view(view))
    return dX, dW


@pytest.mark.parametrize("name", ["C1", "C2", "C3b", "C4", "C5"])
def test_config_parity(name):
    _check(workloads.CONFIGS[name], what=name)


def _small(m, n, r, c, k, p, N, dtype, seed=0):
    return workloads.Config("t", m, n, r, c, k, p, N, dtype, 0.05, seed)


EDGE = [
    (_small(10, 10, 5, 5, 2, 0.5, 1, "f32"), 0),
    (_small(96, 200, 48, 100, 4, 0.2, 7, "f32"), 3),
    (_small(33, 77, 3, 7, 3, 0.3, 9, "bf16"), 0),               # nothing aligned: vector-ALU kernels
    (_small(256, 256, 128, 128, 8, 0.2, 64, "f16"), 0),
    (_small(640, 256, 128, 128, 8, 0.2, 24, "bf16"), 0),        # narrow batch tile, split over m
    (_small(300, 1096, 128, 256, 8, 0.15, 72, "f16"), 0),       # edge tiles
    (_small(130, 200, 65, 100, 40, 0.05, 136, "bf16"), 8),      # padded leading dimensions, rank above 32
    (_small(200, 136, 100, 136, 4, 0.3, 20, "f16"), 0),         # N not a multiple of 8
    (_small(1152, 1024, 576, 512, 145, 0.02, 128, "bf16"), 0),  # the paper's tile shape and a rank it uses
    (_small(768, 256, 384, 128, 40, 0.05, 16, "bf16"), 0),      # slices that start inside a tile, two I_p words
    (_small(1024, 384, 256, 384, 16, 0.1, 40, "f16"), 0),       # workgroups at three offsets inside a tile column
    (_small(512, 128, 128, 128, 64, 0.03, 8, "f16"), 0),        # smallest tile rows of the tuned mask path, rank 64
    (_small(2048, 512, 512, 512, 32, 0.06, 4, "bf16"), 0),      # batch of 4: the tile kernel's 32-column form, mostly idle
    (_small(1024, 640, 256, 128, 16, 0.1, 1, "f16"), 0),        # one column
    (_small(300, 1096, 128, 256, 8, 0.15, 3, "bf16"), 0),       # three columns, edge tiles
    # the pipelined transposed kernel (aligned tiles, batch above 32 columns)
    (_small(256, 256, 128, 128, 8, 0.2, 128, "f16"), 0),        # one panel of four slabs, one 128-row unit per tile row
    (_small(1536, 384, 256, 384, 16, 0.1, 136, "bf16"), 0),     # three panels, three slices, a short second batch block
    (_small(1024, 128, 128, 128, 64, 0.03, 72, "f16"), 0),      # rank 64: two I_p words per row, a batch block of 72
    (_small(768, 256, 384, 128, 40, 0.05, 80, "bf16"), 8),      # rank 40, three units per tile row, padded leading dimensions
    (_small(2048, 256, 512, 256, 5, 0.3, 256, "f16"), 0),       # rank 5 (a short round of ranks), four panels
    (_small(1024, 256, 256, 128, 16, 0.1, 48, "bf16"), 0),      # 33 to 64 batch columns: part of the batch block idle
    # the same kernel on tile widths that are an odd multiple of 64 (Table 2's 576-column tiles): workgroups whose 128
    # columns lie in two tile columns
    (_small(512, 1152, 128, 576, 8, 0.2, 128, "f16"), 0),       # nine workgroups, the fifth across the two tile columns
    (_small(1536, 1152, 512, 576, 40, 0.05, 136, "bf16"), 0),   # two I_p words, three panels, slices, a short batch block
    (_small(1024, 384, 256, 192, 16, 0.1, 72, "f16"), 8),       # 192-column tiles, padded leading dimensions
    (_small(640, 256, 128, 64, 8, 0.2, 128, "bf16"), 0),        # 64-column tiles: every workgroup has two tile columns
    (_small(2048, 1152, 512, 576, 64, 0.04, 256, "f16"), 0),    # rank 64, four panels
    (_small(256, 960, 128, 192, 8, 0.2, 24, "f16"), 0),         # gradient: the last column block's upper half is past the matrix
    (_small(1024, 1152, 512, 576, 32, 0.054, 64, "bf16"), 0),   # gradient: rank 32 on 576-column tiles
]


@pytest.mark.parametrize("idx", range(len(EDGE)))
def test_edge_shapes(idx):
    cfg, ldpad = EDGE[idx]
    _check(cfg, ldpad=ldpad)


def test_without_workspace_the_reduction_is_not_split():
    cfg = _small(2048, 256, 128, 128, 8, 0.2, 32, "f16")
    assert lrbi.masked_gemm_t_workspace_bytes(desc_of(cfg), lrbi.F16, cfg.N) > 0
    a, _ = _check(cfg, use_workspace=True)
    b, _ = _check(cfg, use_workspace=False)
    assert orc.rel_err(to_float64(a), to_float64(b)) <= 1e-2


@pytest.mark.parametrize("N", [16, 128])
def test_nonfinite_values_under_pruned_weights_never_reach_dx(N):
    cfg = _small(256, 512, 128, 256, 8, 0.15, N, "f16")
    data, dYs = _inputs(cfg)
    desc = desc_of(cfg)
    M = orc.decode_mask(data["Ip01"], data["Iz01"], cfg.m, cfg.n, cfg.r, cfg.c, cfg.k)
    Wn = data["W"].copy()
    Wn[M == 0] = np.float16(np.nan)
    Wn[::3][M[::3] == 0] = np.float16(np.inf)
    dIp, dIz = device_factors(desc, data["Ip01"], data["Iz01"])
    dY = to_device(dYs, cfg.dtype)
    a = lrbi.masked_gemm_t(desc, to_device(data["W"], cfg.dtype), dIp, dIz, dY)
    b = lrbi.masked_gemm_t(desc, to_device(Wn, cfg.dtype), dIp, dIz, dY)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
