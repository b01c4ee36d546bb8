"""GPU parity: lrbi_masked_conv3x3 (the masked product of a 3 x 3 convolution, X gathered from the activation)
against the fp64 oracle, and bit for bit against lrbi_masked_gemm on the explicitly unfolded input."""
import numpy as np
import pytest
import torch

import paper_1905_05686_amd as lrbi
import workloads
from oracle import conv as conv_oracle
from oracle import lrbi_oracle as orc
from gpu_util import TOL, desc_of, dev, device_factors, to_device, to_float64

pytestmark = pytest.mark.gpu

DT_CODE = {"f16": lrbi.F16, "bf16": lrbi.BF16}


def _case(m, cin, r, c, k, p, batch, H, Wd, dtype, seed=0):
    cfg = workloads.Config("conv", m, 9 * cin, r, c, k, p, batch * H * Wd, dtype, 0.05, seed)
    rng = np.random.default_rng(seed)
    W = workloads.to_storage(rng.standard_normal((m, 9 * cin), dtype=np.float32) * np.float32(0.05), dtype)
    Ip01, Iz01 = workloads.make_factors(rng, cfg.tiles, r, c, k, p)
    act = workloads.to_storage(rng.standard_normal((batch, H, Wd, cin), dtype=np.float32), dtype)
    return cfg, W, Ip01, Iz01, act


def _padded(act_dev):
    batch, H, Wd, cin = act_dev.shape
    out = torch.zeros((batch, H + 2, Wd + 2, cin), dtype=act_dev.dtype, device=act_dev.device)
    out[:, 1:H + 1, 1:Wd + 1, :] = act_dev
    return out


def _unfold_dev(padded, H, Wd):
    batch, cin = padded.shape[0], padded.shape[3]
    X = torch.empty((9 * cin, batch * H * Wd), dtype=padded.dtype, device=padded.device)
    for kh in range(3):
        for kw in range(3):
            X[(kh * 3 + kw) * cin:(kh * 3 + kw + 1) * cin] = padded[:, kh:kh + H, kw:kw + Wd, :].reshape(-1, cin).T
    return X


SHAPES = [
    # m, cin, r, c, k, p, batch, H, Wd, dtype
    (256, 256, 128, 128, 8, 0.2, 4, 14, 14, "bf16"),    # the ResNet configuration's layer at a small batch: 784 columns
    (128, 128, 128, 384, 6, 0.25, 2, 5, 7, "f16"),      # 70 columns: one partly filled column block
    (256, 128, 128, 384, 16, 0.1, 3, 8, 8, "bf16"),     # tiles three channel blocks wide: slabs cross filter taps
    (128, 128, 128, 1152, 4, 0.3, 1, 1, 1, "f16"),      # a single output pixel (everything but the centre tap is padding)
]


@pytest.mark.parametrize("m,cin,r,c,k,p,batch,H,Wd,dtype", SHAPES)
def test_conv_matches_oracle_and_unfolded_product(m, cin, r, c, k, p, batch, H, Wd, dtype):
    cfg, W, Ip01, Iz01, act = _case(m, cin, r, c, k, p, batch, H, Wd, dtype)
    print("conv", (m, cin, r, c, k, batch, H, Wd, dtype), flush=True)
    desc = desc_of(cfg)
    dIp, dIz = device_factors(desc, Ip01, Iz01)
    dW = to_device(W, dtype)
    dact = _padded(to_device(act.reshape(batch * H * Wd, cin), dtype).reshape(batch, H, Wd, cin))
    wsb = lrbi.masked_conv3x3_workspace_bytes(desc, DT_CODE[dtype], batch, H, Wd)
    ws = torch.empty(max(1, wsb // 4), dtype=torch.float32, device=dev()) if wsb else None
    Y = lrbi.masked_conv3x3(desc, dW, dIp, dIz, dact, workspace=ws)
    torch.cuda.synchronize()
    M = orc.decode_mask(Ip01, Iz01, cfg.m, cfg.n, cfg.r, cfg.c, cfg.k)
    ref = conv_oracle.masked_conv3x3(workloads.to_float64(W, dtype), M, workloads.to_float64(act, dtype))
    err = orc.rel_err(to_float64(Y), ref)
    print("conv rel_err %.3e (tol %.0e)" % (err, TOL[dtype]), flush=True)
    assert err <= TOL[dtype]
    # the same product through the matrix entry point on the unfolded input: same kernel family, same summation
    # order per output, so the bits agree
    X = _unfold_dev(dact, H, Wd)
    if X.shape[1] % 8 == 0:
        gws_b = lrbi.masked_gemm_workspace_bytes(desc, DT_CODE[dtype], X.shape[1])
        gws = torch.empty(max(1, gws_b // 4), dtype=torch.float32, device=dev()) if gws_b else None
        Yg = lrbi.masked_gemm(desc, dW, dIp, dIz, X, workspace=gws)
        assert orc.rel_err(to_float64(Yg), ref) <= TOL[dtype]
        assert float((Y.float() - Yg.float()).abs().max()) <= 2.0 * TOL[dtype] * float(Yg.float().abs().max())


def test_conv_pruned_weights_and_border_never_reach_y():
    m, cin, r, c, k, p, batch, H, Wd, dtype = 128, 128, 128, 384, 6, 0.25, 2, 6, 6, "bf16"
    cfg, W, Ip01, Iz01, act = _case(m, cin, r, c, k, p, batch, H, Wd, dtype, seed=3)
    desc = desc_of(cfg)
    dIp, dIz = device_factors(desc, Ip01, Iz01)
    dact = _padded(to_device(act.reshape(-1, cin), dtype).reshape(batch, H, Wd, cin))
    M = orc.decode_mask(Ip01, Iz01, cfg.m, cfg.n, cfg.r, cfg.c, cfg.k)
    Y = lrbi.masked_conv3x3(desc, to_device(W, dtype), dIp, dIz, dact)
    W32 = workloads.to_float64(W, dtype).astype(np.float32)
    poisoned = workloads.to_storage(np.where(M == 1, W32, np.float32(np.nan)), dtype)
    Yp = lrbi.masked_conv3x3(desc, to_device(poisoned, dtype), dIp, dIz, dact)
    torch.cuda.synchronize()
    assert torch.isfinite(Yp).all() and torch.equal(Y.view(torch.int16), Yp.view(torch.int16))


def test_conv_refuses_shapes_it_cannot_serve():
    cfg, W, Ip01, Iz01, act = _case(128, 64, 128, 192, 4, 0.3, 1, 4, 4, "f16")  # tiles of 192 columns: not a multiple of 128
    desc = desc_of(cfg)
    dIp, dIz = device_factors(desc, Ip01, Iz01)
    dact = _padded(to_device(act.reshape(-1, 64), "f16").reshape(1, 4, 4, 64))
    with pytest.raises(lrbi.LrbiError):
        lrbi.masked_conv3x3(desc, to_device(W, "f16"), dIp, dIz, dact)
