"""The library allocates nothing and never synchronises, so its calls can be captured into a HIP graph.  Each case is
replayed several times with eager work and synchronisations of the test's own in between, and every replay is compared
with the eager result (bit for bit: all kernels sum in a fixed order)."""
import numpy as np
import pytest
import torch

import paper_1905_05686_amd as lrbi
import workloads
from gpu_util import desc_of, dev, device_factors, to_device

pytestmark = pytest.mark.gpu


def _cfg(m, n, r, c, k, dtype, seed, N=16):
    return workloads.Config("t", m, n, r, c, k, 0.15, N, dtype, 0.05, seed)


def _replay_and_compare(run, outputs, scratch):
    """run() writes `outputs` (device tensors).  Eager reference first, then capture, then three replays."""
    run()
    torch.cuda.synchronize()
    ref = [o.clone() for o in outputs]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for rep in range(3):
        for o in outputs:
            o.fill_(0)               # eager work between replays: results must be rewritten by the replay
        scratch.add_(1.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for o, r in zip(outputs, ref):
            a = o.view(torch.uint8) if o.dtype != torch.uint8 else o
            b = r.view(torch.uint8) if r.dtype != torch.uint8 else r
            assert torch.equal(a, b), "replay %d differs from the eager result" % rep


def test_threshold_search_in_a_graph():
    cfg = _cfg(256, 512, 128, 256, 16, "f16", 1)
    d = desc_of(cfg)
    data = workloads.make(cfg, want_x=False)
    f = workloads.make_real_factors(cfg)
    W = to_device(data["W"], cfg.dtype)
    Mp, Mz = torch.from_numpy(f["Mp"]).to(dev()), torch.from_numpy(f["Mz"]).to(dev())
    ws = torch.empty(lrbi.search_workspace_bytes(d), dtype=torch.uint8, device=dev())
    T = cfg.tiles
    keep = {}

    def run():
        out = lrbi.search_thresholds(d, W, f["w_threshold"], Mp, Mz, 0.9, [0.5, 0.8, 0.9], 6, 40, want_factors=True,
                                     workspace=ws)
        if not keep:
            keep["out"] = out
        else:  # same buffers on every call so that the graph's outputs are the ones compared
            for dst, src in zip(keep["out"], out):
                dst.copy_(src)

    # the binding allocates its outputs; for a graph they must be fixed, so call once and reuse through copies
    run()
    outs = list(keep["out"])
    _replay_and_compare(run, outs, torch.zeros(8, device=dev()))


def test_nmf_and_lstm_step_in_a_graph():
    cfg = _cfg(256, 512, 128, 128, 8, "f16", 2)
    d = desc_of(cfg)
    data = workloads.make(cfg, want_x=False)
    W = to_device(data["W"], cfg.dtype)
    rng = np.random.default_rng(3)
    Mp0 = torch.from_numpy(rng.uniform(0.1, 1.0, (cfg.tiles, cfg.r, cfg.k)).astype(np.float32)).to(dev())
    Mz0 = torch.from_numpy(rng.uniform(0.1, 1.0, (cfg.tiles, cfg.k, cfg.c)).astype(np.float32)).to(dev())
    Mp, Mz = Mp0.clone(), Mz0.clone()
    nws = torch.empty(lrbi.nmf_workspace_bytes(d), dtype=torch.uint8, device=dev())

    def run_nmf():
        Mp.copy_(Mp0)
        Mz.copy_(Mz0)
        lrbi.nmf(d, W, Mp, Mz, 5, workspace=nws)   # odd: ends with the copy back from the workspace

    _replay_and_compare(run_nmf, [Mp, Mz], torch.zeros(8, device=dev()))

    # LSTM step: m = 4 H rows, the step reads [x; h] and writes h into its lower half
    H, B = cfg.m // 4, 20
    dIp, dIz = device_factors(d, *[workloads.make(cfg, want_w=False, want_x=False)[k_] for k_ in ("Ip01", "Iz01")])
    xh0 = torch.randn((cfg.n, B), device=dev()).to(torch.float16)
    xh = xh0.clone()
    c0 = torch.randn((H, B), device=dev())
    c = c0.clone()
    hout = torch.empty((H, B), dtype=torch.float16, device=dev())
    lws = torch.empty(lrbi.lstm_step_workspace_bytes(d, lrbi.F16, B), dtype=torch.uint8, device=dev())

    def run_lstm():
        xh.copy_(xh0)
        c.copy_(c0)
        lrbi.lstm_step(d, W, dIp, dIz, xh, c, hout, None, workspace=lws)

    _replay_and_compare(run_lstm, [c, hout], torch.zeros(8, device=dev()))
