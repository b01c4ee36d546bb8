"""GPU parity on the LSTM configuration: 2 layers x 35 steps of sequential masked
products.  The cell equations are the builder's (the paper prints none), so the
graded comparison is the teacher-forced one: every product gets the oracle's own
[x; h] input (rounded to fp16) and is compared with the oracle's pre-activation."""
import numpy as np
import pytest
import torch

import paper_1905_05686_amd as lrbi
import workloads
from oracle import lrbi_oracle as orc
from oracle import lstm as lstm_oracle
from gpu_util import ORACLE_THREADS, TOL, desc_of, device_factors, to_device, to_float64, workspace_for

pytestmark = pytest.mark.gpu


def _round_f16(a):
    return a.astype(np.float16).astype(np.float64)


def test_lstm_teacher_forced_and_free_running():
    L = workloads.make_lstm()
    cfg = L["cfg"]
    H, B, steps, layers = L["hidden"], L["batch"], L["steps"], L["layers"]
    Ws64 = [workloads.to_float64(w, cfg.dtype) for w in L["W"]]
    Ms = [orc.decode_mask(L["Ip01"][l], L["Iz01"][l], cfg.m, cfg.n, cfg.r, cfg.c, cfg.k) for l in range(layers)]
    xs64 = workloads.to_float64(L["x"], cfg.dtype)
    print("lstm oracle...", flush=True)
    ref = lstm_oracle.lstm_sequence(Ws64, Ms, xs64, round_input=_round_f16, threads=ORACLE_THREADS)

    desc = desc_of(cfg)
    dW = [to_device(w, cfg.dtype) for w in L["W"]]
    fac = [device_factors(desc, L["Ip01"][l], L["Iz01"][l]) for l in range(layers)]
    ws = workspace_for(desc, lrbi.F16, B)

    # teacher-forced: 70 products, each against the oracle's pre-activation
    print("lstm teacher-forced...", flush=True)
    worst = 0.0
    for t in range(steps):
        for l in range(layers):
            xh = torch.from_numpy(ref["xh"][t][l].astype(np.float16)).cuda()
            z = lrbi.masked_gemm(desc, dW[l], fac[l][0], fac[l][1], xh, workspace=ws)
            worst = max(worst, orc.rel_err(to_float64(z), ref["z"][t][l]))
    print("lstm teacher-forced worst rel_err %.3e" % worst, flush=True)
    assert worst <= TOL["f16"]

    # free-running: the GPU feeds its own fp16 h forward; gates are harness code (torch)
    print("lstm free-running...", flush=True)
    xs = to_device(L["x"], cfg.dtype)
    h = [torch.zeros((H, B), dtype=torch.float32, device="cuda") for _ in range(layers)]
    c = [torch.zeros((H, B), dtype=torch.float32, device="cuda") for _ in range(layers)]
    for t in range(steps):
        x = xs[t]
        for l in range(layers):
            xh = torch.cat([x, h[l].to(torch.float16)], dim=0)
            z = lrbi.masked_gemm(desc, dW[l], fac[l][0], fac[l][1], xh, workspace=ws).float()
            zi, zf, zg, zo = z[0:H], z[H:2 * H], z[2 * H:3 * H], z[3 * H:4 * H]
            c[l] = torch.sigmoid(zf) * c[l] + torch.sigmoid(zi) * torch.tanh(zg)
            h[l] = torch.sigmoid(zo) * torch.tanh(c[l])
            x = h[l].to(torch.float16)
    for l in range(layers):
        eh = orc.rel_err(to_float64(h[l]), ref["h"][l])
        ec = orc.rel_err(to_float64(c[l]), ref["c"][l])
        print("lstm free-running layer %d: h err %.3e, c err %.3e" % (l, eh, ec), flush=True)
        assert eh <= 1e-2 and ec <= 1e-2


def test_fused_lstm_step_against_the_oracle():
    """lrbi_lstm_step: gate product + cell equations in two launches, h written straight into the next inputs.
    Teacher-forced single steps (oracle's inputs and cell state in, c_t and h_t compared), then the whole
    free-running 2 x 35 sequence through the entry point alone."""
    L = workloads.make_lstm()
    cfg = L["cfg"]
    H, B, steps, layers = L["hidden"], L["batch"], L["steps"], L["layers"]
    Ws64 = [workloads.to_float64(w, cfg.dtype) for w in L["W"]]
    Ms = [orc.decode_mask(L["Ip01"][l], L["Iz01"][l], cfg.m, cfg.n, cfg.r, cfg.c, cfg.k) for l in range(layers)]
    xs64 = workloads.to_float64(L["x"], cfg.dtype)
    ref = lstm_oracle.lstm_sequence(Ws64, Ms, xs64, round_input=_round_f16, threads=ORACLE_THREADS)
    desc = desc_of(cfg)
    dW = [to_device(w, cfg.dtype) for w in L["W"]]
    fac = [device_factors(desc, L["Ip01"][l], L["Iz01"][l]) for l in range(layers)]
    ws = torch.empty(lrbi.lstm_step_workspace_bytes(desc, lrbi.F16, B), dtype=torch.uint8, device="cuda")

    def sigm(z):
        return 1.0 / (1.0 + np.exp(-z))

    # teacher-forced: a few (step, layer) pairs; the expected c_t, h_t follow from the oracle's z and a c_{t-1} of our own
    rng = np.random.default_rng(3)
    for (t, l) in [(0, 0), (1, 1), (17, 0), (34, 1)]:
        xh = torch.from_numpy(ref["xh"][t][l].astype(np.float16)).cuda()
        c_prev = rng.standard_normal((H, B)).astype(np.float32)
        C = torch.from_numpy(c_prev.copy()).cuda()
        h1 = torch.empty((H, B), dtype=torch.float16, device="cuda")
        h2 = torch.empty((H, B), dtype=torch.float16, device="cuda")
        lrbi.lstm_step(desc, dW[l], fac[l][0], fac[l][1], xh, C, h1, h2, workspace=ws)
        torch.cuda.synchronize()
        z = ref["z"][t][l]
        c_ref = sigm(z[H:2 * H]) * c_prev.astype(np.float64) + sigm(z[0:H]) * np.tanh(z[2 * H:3 * H])
        h_ref = sigm(z[3 * H:4 * H]) * np.tanh(c_ref)
        ec, eh = orc.rel_err(to_float64(C), c_ref), orc.rel_err(to_float64(h1), h_ref)
        print("fused step (t=%d, layer %d): c err %.3e, h err %.3e" % (t, l, ec, eh), flush=True)
        assert ec <= 1e-2 and eh <= 1e-2 and torch.equal(h1, h2)

    # free-running: per layer one [2H, B] input buffer; a step reads it and writes h_t into its lower half and into
    # the next layer's upper half
    xs = to_device(L["x"], cfg.dtype)
    xh = [torch.zeros((2 * H, B), dtype=torch.float16, device="cuda") for _ in range(layers)]
    c = [torch.zeros((H, B), dtype=torch.float32, device="cuda") for _ in range(layers)]
    last = torch.empty((H, B), dtype=torch.float16, device="cuda")
    for t in range(steps):
        xh[0][:H].copy_(xs[t])
        for l in range(layers):
            nxt = xh[l + 1][:H] if l + 1 < layers else None
            lrbi.lstm_step(desc, dW[l], fac[l][0], fac[l][1], xh[l], c[l], xh[l][H:], nxt, workspace=ws)
    torch.cuda.synchronize()
    for l in range(layers):
        eh = orc.rel_err(to_float64(xh[l][H:]), ref["h"][l])
        ec = orc.rel_err(to_float64(c[l]), ref["c"][l])
        print("fused free-running layer %d: h err %.3e, c err %.3e" % (l, eh, ec), flush=True)
        assert eh <= 1e-2 and ec <= 1e-2


def test_lstm_step_single_kernel_form():
    """When h does not go into the buffer the step reads, product and cell equations run as one kernel (a workgroup
    owns the four gate rows of its hidden units).  Same bits as the two-launch form (forced here by letting the second
    h output alias the input), and the free-running 2 x 35 sequence with alternating input buffers against the oracle."""
    L = workloads.make_lstm()
    cfg = L["cfg"]
    H, B, steps, layers = L["hidden"], L["batch"], L["steps"], L["layers"]
    desc = desc_of(cfg)
    dW = [to_device(w, cfg.dtype) for w in L["W"]]
    fac = [device_factors(desc, L["Ip01"][l], L["Iz01"][l]) for l in range(layers)]
    ws = torch.empty(lrbi.lstm_step_workspace_bytes(desc, lrbi.F16, B), dtype=torch.uint8, device="cuda")
    rng = np.random.default_rng(21)
    xh_host = (rng.standard_normal((2 * H, B)) * 0.5).astype(np.float16)
    c_prev = rng.standard_normal((H, B)).astype(np.float32)
    outs = []
    for alias in (False, True):
        xh = torch.from_numpy(xh_host.copy()).cuda()
        C = torch.from_numpy(c_prev.copy()).cuda()
        h1 = torch.full((H, B), 7.0, dtype=torch.float16, device="cuda")
        h2 = xh[:H] if alias else None
        print("lstm single-kernel form, alias", alias, flush=True)
        lrbi.lstm_step(desc, dW[0], fac[0][0], fac[0][1], xh, C, h1, h2, workspace=ws)
        torch.cuda.synchronize()
        outs.append((C.clone(), h1.clone()))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])

    Ws64 = [workloads.to_float64(w, cfg.dtype) for w in L["W"]]
    Ms = [orc.decode_mask(L["Ip01"][l], L["Iz01"][l], cfg.m, cfg.n, cfg.r, cfg.c, cfg.k) for l in range(layers)]
    ref = lstm_oracle.lstm_sequence(Ws64, Ms, workloads.to_float64(L["x"], cfg.dtype), round_input=_round_f16,
                                    threads=ORACLE_THREADS)
    xs = to_device(L["x"], cfg.dtype)
    xh = [[torch.zeros((2 * H, B), dtype=torch.float16, device="cuda") for _ in range(2)] for _ in range(layers)]
    c = [torch.zeros((H, B), dtype=torch.float32, device="cuda") for _ in range(layers)]
    print("lstm single-kernel form, free-running", flush=True)
    for t in range(steps):
        cur, nxt = t % 2, (t + 1) % 2
        xh[0][cur][:H].copy_(xs[t])
        for l in range(layers):
            up = xh[l + 1][cur][:H] if l + 1 < layers else None
            lrbi.lstm_step(desc, dW[l], fac[l][0], fac[l][1], xh[l][cur], c[l], xh[l][nxt][H:], up, workspace=ws)
    torch.cuda.synchronize()
    for l in range(layers):
        eh = orc.rel_err(to_float64(xh[l][steps % 2][H:]), ref["h"][l])
        ec = orc.rel_err(to_float64(c[l]), ref["c"][l])
        print("single-kernel free-running layer %d: h err %.3e, c err %.3e" % (l, eh, ec), flush=True)
        assert eh <= 1e-2 and ec <= 1e-2


@pytest.mark.parametrize("H,n,r,c,k,B,dtype,flags", [
    (64, 128, 64, 64, 4, 20, "f16", lrbi.FLAG_PATH_MFMA),  # tile kernel, one slice: a single plane in the workspace
    (64, 128, 64, 64, 4, 20, "f16", 0),       # the same as one kernel on 16 workgroups
    (300, 600, 1200, 600, 145, 20, "f16", 0),  # a layer of size 300 (Sec. 4), untiled, rank 145 (Table 2): 75 workgroups
    (75, 152, 100, 76, 8, 3, "bf16", 0),      # tiles that fit no tuned kernel, tiny batch, cut-off edge tiles
    (128, 512, 128, 128, 8, 36, "f16", 0),    # tuned product kernel, several slices
    (256, 1024, 256, 256, 16, 128, "bf16", 0),
    # enough rows for the row-streaming kernels, h apart from the input: the step as one kernel
    (512, 520, 256, 130, 6, 12, "bf16", 0),   # a short last slab, tiles cut through mask words, one block of columns
    (512, 512, 128, 128, 8, 32, "f16", 0),    # both blocks of columns; a gate's rows start a tile
    (516, 256, 172, 64, 5, 4, "f16", 0),      # tile height no multiple of 16: the units of a workgroup sit anywhere in a tile
    (510, 256, 170, 64, 5, 8, "f16", 0),      # H and r no multiples of 4: two launches
])
def test_fused_lstm_step_small_shapes(H, n, r, c, k, B, dtype, flags):
    cfg = workloads.Config("t", 4 * H, n, r, c, k, 0.2 if k < 64 else 0.05, B, dtype, 0.1, 5)
    data = workloads.make(cfg)
    desc = desc_of(cfg, flags)
    dIp, dIz = device_factors(desc, data["Ip01"], data["Iz01"])
    rng = np.random.default_rng(9)
    c_prev = rng.standard_normal((H, B)).astype(np.float32)
    C = torch.from_numpy(c_prev.copy()).cuda()
    tdt = torch.float16 if dtype == "f16" else torch.bfloat16
    h1 = torch.empty((H, B), dtype=tdt, device="cuda")
    lrbi.lstm_step(desc, to_device(data["W"], dtype), dIp, dIz, to_device(data["X"], dtype), C, h1)
    torch.cuda.synchronize()
    M = orc.decode_mask(data["Ip01"], data["Iz01"], cfg.m, cfg.n, cfg.r, cfg.c, cfg.k)
    z = orc.masked_gemm(workloads.to_float64(data["W"], dtype), M, workloads.to_float64(data["X"], dtype))
    sg = lambda v: 1.0 / (1.0 + np.exp(-v))
    c_ref = sg(z[H:2 * H]) * c_prev.astype(np.float64) + sg(z[0:H]) * np.tanh(z[2 * H:3 * H])
    h_ref = sg(z[3 * H:]) * np.tanh(c_ref)
    assert orc.rel_err(to_float64(C), c_ref) <= 1e-2 and orc.rel_err(to_float64(h1), h_ref) <= 1e-2


def test_lstm_sequence_on_the_rank_145_layer():
    """An LSTM layer of the size Sec. 4 names (300 units: a 1200 x 600 gate matrix; untiled here, the paper does not say)
    at Table 2's rank 145, 2 layers x 35 steps through lrbi_lstm_step with alternating input buffers, free-running, against the oracle; the
    product runs on the row-streaming kernel with far fewer workgroups than compute units."""
    L = workloads.make_lstm(hidden=300, r=1200, c=600, k=145, p=0.05)
    cfg = L["cfg"]
    H, B, steps, layers = L["hidden"], L["batch"], L["steps"], L["layers"]
    assert (cfg.m, cfg.n, cfg.r, cfg.c, cfg.k) == (1200, 600, 1200, 600, 145)
    Ws64 = [workloads.to_float64(w, cfg.dtype) for w in L["W"]]
    Ms = [orc.decode_mask(L["Ip01"][l], L["Iz01"][l], cfg.m, cfg.n, cfg.r, cfg.c, cfg.k) for l in range(layers)]
    assert 0.2 < Ms[0].mean() < 0.5
    ref = lstm_oracle.lstm_sequence(Ws64, Ms, workloads.to_float64(L["x"], cfg.dtype), round_input=_round_f16,
                                    threads=ORACLE_THREADS)
    desc = desc_of(cfg)
    dW = [to_device(w, cfg.dtype) for w in L["W"]]
    fac = [device_factors(desc, L["Ip01"][l], L["Iz01"][l]) for l in range(layers)]
    ws = torch.empty(max(16, lrbi.lstm_step_workspace_bytes(desc, lrbi.F16, B)), dtype=torch.uint8, device="cuda")
    xs = to_device(L["x"], cfg.dtype)
    xh = [[torch.zeros((2 * H, B), dtype=torch.float16, device="cuda") for _ in range(2)] for _ in range(layers)]
    c = [torch.zeros((H, B), dtype=torch.float32, device="cuda") for _ in range(layers)]
    for t in range(steps):
        cur, nxt = t % 2, (t + 1) % 2
        xh[0][cur][:H].copy_(xs[t])
        for l in range(layers):
            up = xh[l + 1][cur][:H] if l + 1 < layers else None
            lrbi.lstm_step(desc, dW[l], fac[l][0], fac[l][1], xh[l][cur], c[l], xh[l][nxt][H:], up, workspace=ws)
    torch.cuda.synchronize()
    for l in range(layers):
        eh = orc.rel_err(to_float64(xh[l][steps % 2][H:]), ref["h"][l])
        ec = orc.rel_err(to_float64(c[l]), ref["c"][l])
        print("rank-145 layer %d: h err %.3e, c err %.3e" % (l, eh, ec), flush=True)
        assert eh <= 1e-2 and ec <= 1e-2
