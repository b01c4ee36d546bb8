"""lrbi_masked_gemm_static (the entry point that allocates nothing: partial sums in the library's own static
scratch array) against lrbi_masked_gemm with a caller workspace, through the C ABI: identical bits, on two
calls in a row, the second with a smaller input that leaves part of the first call's scratch contents behind."""
import ctypes

import numpy as np
import pytest
import torch

import paper_1905_05686_amd as lrbi
import workloads
from oracle import lrbi_oracle as orc
from gpu_util import TOL, desc_of, dev, device_factors, to_device, workspace_for

pytestmark = pytest.mark.gpu

DC = {"f32": lrbi.F32, "f16": lrbi.F16, "bf16": lrbi.BF16}


def _case(cfg):
    data = workloads.make(cfg)
    d = desc_of(cfg)
    dIp, dIz = device_factors(d, data["Ip01"], data["Iz01"])
    W = to_device(data["W"], cfg.dtype)
    X = to_device(data["X"], cfg.dtype)
    return data, d, dIp, dIz, W, X


def _both(cfg):
    data, d, dIp, dIz, W, X = _case(cfg)
    need = lrbi.masked_gemm_workspace_bytes(d, DC[cfg.dtype], cfg.N)
    ws = workspace_for(d, DC[cfg.dtype], cfg.N)
    ref = lrbi.masked_gemm(d, W, dIp, dIz, X, workspace=ws)
    out = torch.full_like(ref, float("nan"))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    lrbi.masked_gemm_static(d, W, dIp, dIz, X, out)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(out.view(torch.int16 if out.element_size() == 2 else torch.int32),
                       ref.view(torch.int16 if ref.element_size() == 2 else torch.int32)), cfg
    # and, like every product, against the oracle
    M = orc.decode_mask(data["Ip01"], data["Iz01"], cfg.m, cfg.n, cfg.r, cfg.c, cfg.k)
    Y = orc.masked_gemm(workloads.to_float64(data["W"], cfg.dtype), M, workloads.to_float64(data["X"], cfg.dtype),
                        threads=16)
    assert orc.rel_err(out.double().cpu().numpy(), Y) <= TOL[cfg.dtype]
    return need


def test_two_calls_in_a_row_second_smaller():
    print("no-alloc: C2-shaped split product, then a smaller one", flush=True)
    big = workloads.Config("na-big", 2048, 4608, 256, 256, 16, 0.08, 128, "f16", 0.01, 5)     # split over n: scratch used
    small = workloads.Config("na-small", 512, 2048, 128, 128, 8, 0.2, 32, "bf16", 0.03, 6)    # split, fewer planes
    need_big = _both(big)
    need_small = _both(small)
    assert need_big > need_small > 0, (need_big, need_small)
    # a shape that needs no scratch at all goes straight through
    assert _both(workloads.Config("na-none", 512, 512, 128, 128, 8, 0.2, 2048, "bf16", 0.03, 7)) == 0


def test_sizes_beyond_the_scratch_are_refused_before_any_launch():
    # a forced split into 8 slices of 16384 x 128 fp32 partial sums: 64 MiB, beyond the 32 MiB array
    d = lrbi.Desc(16384, 8192, 256, 256, 16, lrbi.flag_splitk(8))
    assert lrbi.masked_gemm_workspace_bytes(d, lrbi.F16, 128) > lrbi.STATIC_SCRATCH_BYTES
    lib = lrbi.load_library()
    p = ctypes.c_void_p(256)     # never dereferenced: the size check comes before any launch
    assert lib.lrbi_masked_gemm_static(ctypes.byref(d), lrbi.F16, p, 8192, p, p, p, 128, 128, p, 128, None) == -8
    assert "workspace" in lrbi.strerror(-8)
