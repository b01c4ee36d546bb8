#!/usr/bin/env python3
"""Benchmark of the LRBI hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input of
configuration C2 (AlexNet 9216->4096 layer: W 4096x9216 fp16, 256x256 tiles,
rank 16, Bernoulli(0.08) factors, X 9216x128): index-size accounting (host),
mask decode to HBM, and the fused masked product that rebuilds the mask in the
kernel.  Inputs are resident in HBM before the timed region.  Weights rotate
over several buffers so that W streams from HBM and not from the 256 MB
last-level cache, as it would inside a network whose layers do not fit there.

Prints ONE JSON line.  `value` is the
dense-equivalent TFLOP/s of the step; the decode part of the metric (Gbit/s on a
mask larger than 1 GiB) and the other configurations ride along as extra keys.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E
MFMA_PEAK_TFLOPS = 2500.0   # dense bf16 / fp16


def _die_multi_gpu(n):
    print("bench.py measures one GPU: this build has no multi-GPU path (the kernels shard by tile "
          "rows without any exchange step); --gpus %d is not supported." % n, file=sys.stderr)
    sys.exit(2)


# kernels behind lrbi_decode_and_gemm on the headline workload; the recorded HBM traffic is only quoted when it was
# measured on these same kernels
C2_GEMM_KERNELS = "mfma_gemm_pipe_kernel (mask stored) + splitk_reduce_kernel"


def _recorded_traffic():
    """HBM bytes per launch of the C2 decode + fused product (kernel + split-K reduction), from the rocprofv3
    FETCH_SIZE / WRITE_SIZE runs summarised under profiles/ (counters cannot be read from inside
    this process); None when no summary is there or when it was taken on other kernels."""
    path = os.path.join(ROOT, "profiles", "C2_masked_gemm_hbm_traffic.md")
    kernels, traffic = None, None
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("kernels:"):
                    kernels = line.split(":", 1)[1].strip()
                if line.startswith("traffic_bytes_per_launch:"):
                    traffic = int(line.split(":")[1].strip())
    except OSError:
        return None
    return traffic if kernels == C2_GEMM_KERNELS else None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-others", action="store_true", help="skip the per-configuration extras")
    ap.add_argument("--extras", default="all",
                    help="comma-separated subset of the extras to run (decode_scaled_C2, decode_scaled_C3, C3a, C3b, "
                         "C4, C5, conv_C5, C1, general_resnet_tiles, general_edge_tiles, paper_fc5_tiles, steady_state_C3_tiles, alg1_eval_C2, alg1_eval_C3, alg1_eval_C4, alg1_eval_paper_fc5_tiles, alg1_search_C2, backward_C2, backward_C3b, backward_paper_fc5_tiles, lstm_sequence_C4, lstm_sequence_paper_rank145, nmf_C2, nmf_C3, nmf_C4, nmf_paper_fc5_tiles, "
                         "ceilings); used to profile one workload at a time")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="for `rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE`: run a plain 1 GiB device copy "
                         "(calibration of the counter) and the C2 fused product on HBM-cold weights, then exit")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        _die_multi_gpu(max(args.gpus, int(os.environ.get("WORLD_SIZE", "1"))))

    import numpy as np
    import torch

    import paper_1905_05686_amd as lrbi
    import workloads

    lrbi.load_library()  # raises if the HIP library has not been built
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    TD = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
    DC = {"f32": lrbi.F32, "f16": lrbi.F16, "bf16": lrbi.BF16}

    def to_dev(a, dtype):
        if dtype == "bf16":
            return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(a).to(dev)

    def factors_to_dev(desc, Ip01, Iz01):
        ip, iz = lrbi.pack_factors(desc, Ip01, Iz01)
        return torch.from_numpy(ip.view(np.int32)).to(dev), torch.from_numpy(iz.view(np.int64)).to(dev)

    def rotated_weights(W, min_total_bytes=600e6):
        """Enough independent copies of W that one round trip exceeds the last-level cache."""
        nbytes = W.numel() * W.element_size()
        copies = min(12, max(2, int(np.ceil(min_total_bytes / nbytes))))
        out = [W]
        for i in range(1, copies):
            out.append(torch.roll(W, shifts=i, dims=0).contiguous())  # same values, different rows/addresses
        return out

    def event_times(fn_list, iters, warmup):
        """Average GPU milliseconds per launch of fn (rotating over fn_list).  The launches are
        captured into one HIP graph and replayed, so that the host's per-call overhead (Python,
        ctypes) does not sit between kernels; HIP events on the launch stream bracket the replay."""
        for i in range(warmup):
            fn_list[i % len(fn_list)]()
        torch.cuda.synchronize()
        try:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for i in range(iters):
                    fn_list[i % len(fn_list)]()
            graph.replay()
            torch.cuda.synchronize()
            ts = []
            for _ in range(3):
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                e0.record()
                graph.replay()
                e1.record()
                torch.cuda.synchronize()
                ts.append(e0.elapsed_time(e1) / iters)
            del graph
            return float(np.mean(ts)), float(sorted(ts)[1])
        except Exception:
            torch.cuda.synchronize()
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(iters):
                fn_list[i % len(fn_list)]()
            e1.record()
            torch.cuda.synchronize()
            t = e0.elapsed_time(e1) / iters
            return float(t), float(t)

    # ------------------------------------------------------------------ headline: C2
    cfg = workloads.CONFIGS["C2"]
    data = workloads.make(cfg)
    desc = lrbi.Desc(cfg.m, cfg.n, cfg.r, cfg.c, cfg.k)
    dIp, dIz = factors_to_dev(desc, data["Ip01"], data["Iz01"])
    Ws = rotated_weights(to_dev(data["W"], cfg.dtype))
    X = to_dev(data["X"], cfg.dtype)
    Y = torch.empty((cfg.m, cfg.N), dtype=TD[cfg.dtype], device=dev)
    mask = torch.empty((cfg.m, ((cfg.n + 127) // 128) * 16), dtype=torch.uint8, device=dev)
    ws_bytes = lrbi.masked_gemm_workspace_bytes(desc, DC[cfg.dtype], cfg.N)
    ws = torch.empty(max(1, (ws_bytes + 3) // 4), dtype=torch.float32, device=dev) if ws_bytes else None

    if args.traffic_probe:
        src = torch.full((1 << 30,), 1, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        for i in range(2 * len(Ws)):
            lrbi.decode_and_gemm(desc, Ws[i % len(Ws)], dIp, dIz, X, out=Y, mask=mask, workspace=ws)
        torch.cuda.synchronize()
        print(json.dumps({"traffic_probe": True, "copy_bytes_each_way": 1 << 30, "copies": 3,
                          "gemm_launches": 2 * len(Ws)}))
        return

    def gpu_step(i):
        # rows a1-a6 in one call: the mask to HBM and the fused masked product (for this shape one product launch,
        # which stores the mask bytes it rebuilds, plus the split reduction)
        lrbi.decode_and_gemm(desc, Ws[i % len(Ws)], dIp, dIz, X, out=Y, mask=mask, workspace=ws)

    for i in range(args.warmup):
        lrbi.index_bits(desc)
        gpu_step(i)
    torch.cuda.synchronize()
    # The GPU part of the K steps is captured once into a HIP graph (decode + fused product of every
    # step, weights rotating) and replayed inside the timed region; the host part of every step
    # (index-size accounting) runs in the timed region as well.
    launch_mode = "hipgraph"
    try:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for i in range(args.steps):
                gpu_step(i)
        graph.replay()  # untimed: first replay uploads the graph
        torch.cuda.synchronize()
    except Exception as e:
        graph = None
        launch_mode = "eager (graph capture failed: %r)" % (e,)
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        lrbi.index_bits(desc)
    if graph is not None:
        graph.replay()
    else:
        for i in range(args.steps):
            gpu_step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    flops = 2.0 * cfg.m * cfg.n * cfg.N
    value = flops / (ms_per_step * 1e-3) / 1e12

    # dominant kernel: the fused product that also leaves the mask, same launch configuration, weights rotating
    gemm_ms, _ = event_times([(lambda Wi=Wi: lrbi.decode_and_gemm(desc, Wi, dIp, dIz, X, out=Y, mask=mask, workspace=ws))
                              for Wi in Ws], 10 * len(Ws), 2 * len(Ws))
    es = 2
    factor_bytes = lrbi.index_bits(desc)["lrbi_bits"] / 8
    # W, X, the packed factors read once; Y and the one-bit-per-weight mask written once
    gemm_bytes = cfg.m * cfg.n * es + cfg.n * cfg.N * es + cfg.m * cfg.N * es + factor_bytes + cfg.m * cfg.n / 8
    achieved = gemm_bytes / (gemm_ms * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": "lrbi_decode_and_gemm (%s)" % C2_GEMM_KERNELS,
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": _recorded_traffic(),
                "avg_launch_ms": round(gemm_ms, 5), "algorithmic_bytes": int(gemm_bytes),
                "tflops_dense_equiv": round(flops / (gemm_ms * 1e-3) / 1e12, 1),
                "mfma_frac": round(flops / (gemm_ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS, 4)}

    # for comparison: the two entry points on their own (the step above no longer launches the decode kernel)
    dec_ms, _ = event_times([lambda: lrbi.decode_mask(desc, dIp, dIz, out=mask)], 100, 10)
    plain_ms, _ = event_times([(lambda Wi=Wi: lrbi.masked_gemm(desc, Wi, dIp, dIz, X, out=Y, workspace=ws)) for Wi in Ws],
                              10 * len(Ws), 2 * len(Ws))

    out = {
        "metric": "mask decode Gbit/s + fused masked-GEMM TFLOP/s (dense-equiv), % of roofline",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic", "launch": launch_mode,
        "config": {"workload": "C2: W 4096x9216 fp16 N(0,0.01), tiles 256x256, rank 16, factors Bernoulli(0.08), "
                               "X 9216x128; step = index_bits + decode_and_gemm (mask to HBM and fused masked product); "
                               "W rotated over %d buffers (HBM-cold)" % len(Ws)},
        "value_note": "dense-equivalent 2*m*n*N flops over the whole step (mask decoded to HBM + fused product)",
        "roofline": roofline,
        "separate_calls": {"mask_bits": cfg.m * cfg.n, "decode_mask_avg_launch_ms": round(dec_ms, 5),
                           "decode_mask_gbit_s": round(cfg.m * cfg.n / (dec_ms * 1e-3) / 1e9, 1),
                           "masked_gemm_avg_launch_ms": round(plain_ms, 5)},
    }

    # ------------------------------------------------------------------ extras
    wanted = None if args.extras == "all" else set(x for x in args.extras.split(",") if x)
    if not args.no_others:
        others = {}
        # decode on masks above 1 GiB (tile shape, rank and p of C2 and of C3), factors drawn on the device
        gen = torch.Generator(device=dev)
        gen.manual_seed(0)
        weights = (2 ** torch.arange(32, device=dev, dtype=torch.int64))

        def packed_bernoulli(rows, bits_per_row, words_per_row, prob):
            outw = torch.zeros((rows, words_per_row), dtype=torch.int32, device=dev)
            chunk = 1 << 20
            for lo in range(0, rows, chunk):
                hi = min(rows, lo + chunk)
                for w in range(words_per_row):
                    nb = min(32, bits_per_row - 32 * w)
                    if nb <= 0:
                        continue
                    b = (torch.rand((hi - lo, nb), device=dev, generator=gen) < prob).to(torch.int64)
                    v = (b * weights[:nb]).sum(dim=1)
                    outw[lo:hi, w] = torch.where(v >= 2 ** 31, v - 2 ** 32, v).to(torch.int32)
            return outw

        for key, base, big_m, big_n in (("decode_scaled_C2", "C2", 65536, 147456), ("decode_scaled_C3", "C3a", 65536, 131072)):
            if wanted is not None and key not in wanted:
                continue
            try:
                big = workloads.scaled(workloads.CONFIGS[base], m=big_m, n=big_n)
                bdesc = lrbi.Desc(big.m, big.n, big.r, big.c, big.k)
                sizes = lrbi.index_bits(bdesc)
                T = big.tiles
                bIp = packed_bernoulli(T * big.r, big.k, (big.k + 31) // 32, big.p)
                bIz = packed_bernoulli(T * big.k, big.c, 2 * ((big.c + 63) // 64), big.p)
                assert bIp.numel() * 4 == sizes["packed_ip_bytes"] and bIz.numel() * 4 == sizes["packed_iz_bytes"]
                bmask = torch.empty((big.m, big.n // 8), dtype=torch.uint8, device=dev)
                ms, med = event_times([lambda: lrbi.decode_mask(bdesc, bIp, bIz, out=bmask)], 10, 3)
                mask_bytes = big.m * big.n / 8
                moved = mask_bytes + sizes["lrbi_bits"] / 8  # the mask written once, the packed factors read once
                others[key] = {
                    "workload": "%s tile shape (%dx%d, rank %d, p=%.2f) on a %dx%d mask (%.2f GiB)" % (
                        base[:2], big.r, big.c, big.k, big.p, big.m, big.n, mask_bytes / 2 ** 30),
                    "avg_launch_ms": round(ms, 4), "gbit_s": round(big.m * big.n / (ms * 1e-3) / 1e9, 1),
                    "write_GBs": round(mask_bytes / (ms * 1e-3) / 1e9, 1),
                    "hbm_frac_on_mask_bytes_written": round(mask_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                    "algorithmic_bytes": int(moved), "GBs": round(moved / (ms * 1e-3) / 1e9, 1),
                    "hbm_frac": round(moved / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
                del bIp, bIz, bmask
            except Exception as e:  # keep the headline line even if an extra fails
                others[key] = {"error": repr(e)}

        # generality of the format: the paper's own 576 x 512 tiles at rank 145 (tiles divide: tuned decode, general
        # product kernel), and the C2 layer grown by a few rows and columns so that its edge tiles are cut off
        # (general kernels throughout)
        general = {
            "general_resnet_tiles": workloads.Config("general_resnet_tiles", 2304, 2048, 576, 512, 145, 0.02, 128, "bf16", 0.02),
            "general_edge_tiles": workloads.Config("general_edge_tiles", 4100, 9224, 256, 256, 16, 0.08, 128, "f16", 0.01),
            # C2's layer in the tiling the paper itself uses for it (Table 2, note 2: 16 x 8 blocks of 576 x 512, here
            # with the 9216 inputs along the columns, so tiles of 512 x 576; rank 32; p for a mask density of 0.09)
            "paper_fc5_tiles": workloads.Config("paper_fc5_tiles", 4096, 9216, 512, 576, 32, 0.054, 128, "f16", 0.01),
        }
        # the C3 tile shape on a product large enough that the prologue and the last partial wave of workgroups do not
        # count: the matrix-core kernel's steady state
        steady = {"steady_state_C3_tiles": workloads.Config("steady_state_C3_tiles", 16384, 16384, 512, 512, 32, 0.06, 4096, "bf16", 0.01)}
        for name in ("C3a", "C3b", "C4", "C5", "C1", "general_resnet_tiles", "general_edge_tiles", "paper_fc5_tiles",
                     "steady_state_C3_tiles"):
            if wanted is not None and name not in wanted:
                continue
            try:
                c = workloads.CONFIGS.get(name) or general.get(name) or steady[name]
                d = workloads.make(c)
                de = lrbi.Desc(c.m, c.n, c.r, c.c, c.k)
                ip_, iz_ = factors_to_dev(de, d["Ip01"], d["Iz01"])
                Wl = rotated_weights(to_dev(d["W"], c.dtype))
                X_ = to_dev(d["X"], c.dtype)
                Y_ = torch.empty((c.m, c.N), dtype=TD[c.dtype], device=dev)
                wb = lrbi.masked_gemm_workspace_bytes(de, DC[c.dtype], c.N)
                w_ = torch.empty(max(1, (wb + 3) // 4), dtype=torch.float32, device=dev) if wb else None
                fns = [(lambda Wi=Wi: lrbi.masked_gemm(de, Wi, ip_, iz_, X_, out=Y_, workspace=w_)) for Wi in Wl]
                ms, med = event_times(fns, 6 * len(fns), len(fns))
                ms_warm, _ = event_times(fns[:1], 40, 5)
                esz = 4 if c.dtype == "f32" else 2
                byts = (c.m * c.n + c.n * c.N + c.m * c.N) * esz + lrbi.index_bits(de)["lrbi_bits"] / 8
                fl = 2.0 * c.m * c.n * c.N
                extra = {}
                if name == "C4":
                    # the whole LSTM sequence's products: 2 layers x 35 steps, each layer's gate matrix reused every step
                    # (so it is served by the last-level cache after the first step), one graph replay of 70 calls
                    seq = [fns[i % 2] for i in range(70)]
                    ms_seq, _ = event_times(seq, 70, 4)
                    extra = {"sequence_70_products_ms": round(ms_seq * 70, 4)}
                if name in general:
                    gmask = torch.empty((c.m, ((c.n + 127) // 128) * 16), dtype=torch.uint8, device=dev)
                    ms_dec, _ = event_times([lambda: lrbi.decode_mask(de, ip_, iz_, out=gmask)], 20, 3)
                    dfns = [(lambda Wi=Wi: lrbi.decode_and_gemm(de, Wi, ip_, iz_, X_, out=Y_, mask=gmask, workspace=w_))
                            for Wi in Wl]
                    ms_both, _ = event_times(dfns, 6 * len(dfns), len(dfns))
                    extra = {"shape": "W %dx%d, tiles %dx%d, rank %d" % (c.m, c.n, c.r, c.c, c.k),
                             "decode_ms": round(ms_dec, 5), "decode_gbit_s": round(c.m * c.n / (ms_dec * 1e-3) / 1e9, 1),
                             "decode_and_gemm_ms_cold": round(ms_both, 5)}
                    del gmask
                others[name] = {"N": c.N, "dtype": c.dtype, "avg_launch_ms_cold": round(ms, 5), **extra,
                                "avg_launch_ms_warm": round(ms_warm, 5),
                                "tflops_dense_equiv": round(fl / (ms * 1e-3) / 1e12, 2),
                                "mfma_frac": round(fl / (ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS, 4),
                                "GBs": round(byts / (ms * 1e-3) / 1e9, 1),
                                "hbm_frac": round(byts / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
                del Wl, X_, Y_
            except Exception as e:
                others[name] = {"error": repr(e)}
        # the convolution configuration without its unfolded input: C5's layer (256 filters, 256 channels, 3 x 3,
        # 14 x 14 images, batch 64) with X gathered from the zero-padded activation inside the product kernel
        if wanted is None or "conv_C5" in wanted:
            try:
                c = workloads.CONFIGS["C5"]
                cin, Hh, Ww = c.n // 9, 14, 14
                batch = c.N // (Hh * Ww)
                d = workloads.make(c, want_x=False)
                de = lrbi.Desc(c.m, c.n, c.r, c.c, c.k)
                ip_, iz_ = factors_to_dev(de, d["Ip01"], d["Iz01"])
                Wl = rotated_weights(to_dev(d["W"], c.dtype), min_total_bytes=8e6)
                acts = []
                for i in range(8):  # rotating activations: each launch reads one that the cache saw 7 launches ago
                    a_ = torch.zeros((batch, Hh + 2, Ww + 2, cin), dtype=TD[c.dtype], device=dev)
                    a_[:, 1:Hh + 1, 1:Ww + 1, :] = torch.randn((batch, Hh, Ww, cin), device=dev, dtype=torch.float32).to(TD[c.dtype])
                    acts.append(a_)
                Y_ = torch.empty((c.m, c.N), dtype=TD[c.dtype], device=dev)
                wb = lrbi.masked_conv3x3_workspace_bytes(de, DC[c.dtype], batch, Hh, Ww)
                w_ = torch.empty(max(1, (wb + 3) // 4), dtype=torch.float32, device=dev) if wb else None
                fns = [(lambda Wi=Wl[i % len(Wl)], Ai=acts[i]: lrbi.masked_conv3x3(de, Wi, ip_, iz_, Ai, out=Y_, workspace=w_))
                       for i in range(len(acts))]
                ms, _ = event_times(fns, 6 * len(fns), len(fns))
                byts = (c.m * c.n + batch * Hh * Ww * cin + c.m * c.N) * 2 + lrbi.index_bits(de)["lrbi_bits"] / 8
                fl = 2.0 * c.m * c.n * c.N
                others["conv_C5"] = {
                    "workload": "C5 as a convolution: %d filters x %d channels x 3 x 3 (%s), images %d x %d x %d, tiles %dx%d "
                                "rank %d; X gathered from the padded activation" % (c.m, cin, c.dtype, batch, Hh, Ww, c.r, c.c, c.k),
                    "avg_launch_ms": round(ms, 5), "tflops_dense_equiv": round(fl / (ms * 1e-3) / 1e12, 2),
                    "mfma_frac": round(fl / (ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS, 4),
                    "algorithmic_bytes": int(byts), "GBs": round(byts / (ms * 1e-3) / 1e9, 1),
                    "hbm_frac": round(byts / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
                del Wl, acts, Y_
            except Exception as e:
                others["conv_C5"] = {"error": repr(e)}
        # one candidate of Algorithm 1 per launch (threshold, decode on chip, ones and cost per tile)
        for name in ("C2", "C3a", "C4", "paper_fc5_tiles"):
            key = "alg1_eval_" + (name[:2] if name in workloads.CONFIGS else name)
            if wanted is not None and key not in wanted:
                continue
            try:
                c = workloads.CONFIGS.get(name) or general[name]
                d = workloads.make(c, want_x=False)
                f = workloads.make_real_factors(c)
                de = lrbi.Desc(c.m, c.n, c.r, c.c, c.k)
                Wl = rotated_weights(to_dev(d["W"], c.dtype))
                tens = [torch.from_numpy(f[k_]).to(dev) for k_ in ("Mp", "Mz", "Tp", "Tz")]
                res = (torch.empty(c.tiles, dtype=torch.int64, device=dev), torch.empty(c.tiles, dtype=torch.float64, device=dev))
                wsb = lrbi.threshold_eval_workspace_bytes(de)
                ews = torch.empty(max(1, wsb // 8), dtype=torch.int64, device=dev) if wsb else None
                fns = [(lambda Wi=Wi: lrbi.threshold_eval(de, Wi, f["w_threshold"], *tens, out=res, workspace=ews))
                       for Wi in Wl]
                ms, _ = event_times(fns, 6 * len(fns), len(fns))
                byts = c.m * c.n * 2 + c.tiles * c.k * (c.r + c.c) * 4 + c.tiles * 16
                others[key] = {"workload": "%s: W %dx%d %s, tiles %dx%d rank %d, U(0,1) factors thresholded at 1 - p, cost threshold 1.645 sigma"
                                           % (key[10:], c.m, c.n, c.dtype, c.r, c.c, c.k),
                               "avg_launch_ms_cold": round(ms, 5), "GBs": round(byts / (ms * 1e-3) / 1e9, 1),
                               "hbm_frac": round(byts / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                               "candidates_per_s": round(1.0 / (ms * 1e-3), 1)}
                del Wl, tens
            except Exception as e:
                others[key] = {"error": repr(e)}
        # the LSTM configuration as a sequence: 2 layers x 35 fused steps (gate product + cell equations, h written
        # straight into the next inputs), one graph replay.  With two input buffers per layer in turn, h never goes
        # into the buffer the step reads and a step is one kernel; with one buffer per layer it is two launches.
        # Against the same sequence with separate product, reduction and (torch) gate kernels
        # (and on a layer of the size Sec. 4 names for its LSTM, 300 units: a 1200 x 600 gate matrix, untiled, at
        # Table 2's rank 145)
        for lkey, lkw in (("lstm_sequence_C4", {}),
                          ("lstm_sequence_paper_rank145", {"hidden": 300, "r": 1200, "c": 600, "k": 145, "p": 0.05})):
            if wanted is not None and lkey not in wanted:
                continue
            try:
                Ld = workloads.make_lstm(**lkw)
                c = Ld["cfg"]
                Hh, Bb, steps_, layers_ = Ld["hidden"], Ld["batch"], Ld["steps"], Ld["layers"]
                de = lrbi.Desc(c.m, c.n, c.r, c.c, c.k)
                Wd = [to_dev(w, c.dtype) for w in Ld["W"]]
                fac = [factors_to_dev(de, Ld["Ip01"][l], Ld["Iz01"][l]) for l in range(layers_)]
                xs_ = to_dev(Ld["x"], c.dtype)
                lws = torch.empty(lrbi.lstm_step_workspace_bytes(de, DC[c.dtype], Bb), dtype=torch.uint8, device=dev)
                xh = [torch.zeros((2 * Hh, Bb), dtype=TD[c.dtype], device=dev) for _ in range(layers_)]
                cs = [torch.zeros((Hh, Bb), dtype=torch.float32, device=dev) for _ in range(layers_)]

                xh2 = [[torch.zeros((2 * Hh, Bb), dtype=TD[c.dtype], device=dev) for _ in range(2)] for _ in range(layers_)]

                def fused_sequence():
                    for t in range(steps_):
                        cur, nx = t % 2, (t + 1) % 2
                        xh2[0][cur][:Hh].copy_(xs_[t])
                        for l in range(layers_):
                            up = xh2[l + 1][cur][:Hh] if l + 1 < layers_ else None
                            lrbi.lstm_step(de, Wd[l], fac[l][0], fac[l][1], xh2[l][cur], cs[l], xh2[l][nx][Hh:], up,
                                           workspace=lws)

                def two_launch_sequence():
                    for t in range(steps_):
                        xh[0][:Hh].copy_(xs_[t])
                        for l in range(layers_):
                            nxt = xh[l + 1][:Hh] if l + 1 < layers_ else None
                            lrbi.lstm_step(de, Wd[l], fac[l][0], fac[l][1], xh[l], cs[l], xh[l][Hh:], nxt, workspace=lws)

                gwb = lrbi.masked_gemm_workspace_bytes(de, DC[c.dtype], Bb)
                gws = torch.empty(max(1, (gwb + 3) // 4), dtype=torch.float32, device=dev) if gwb else None
                zbuf = torch.empty((c.m, Bb), dtype=TD[c.dtype], device=dev)

                def unfused_sequence():
                    for t in range(steps_):
                        xh[0][:Hh].copy_(xs_[t])
                        for l in range(layers_):
                            z = lrbi.masked_gemm(de, Wd[l], fac[l][0], fac[l][1], xh[l], out=zbuf, workspace=gws).float()
                            cs[l].copy_(torch.sigmoid(z[Hh:2 * Hh]) * cs[l] + torch.sigmoid(z[0:Hh]) * torch.tanh(z[2 * Hh:3 * Hh]))
                            hcur = (torch.sigmoid(z[3 * Hh:]) * torch.tanh(cs[l])).to(TD[c.dtype])
                            xh[l][Hh:].copy_(hcur)
                            if l + 1 < layers_:
                                xh[l + 1][:Hh].copy_(hcur)

                ms_f, _ = event_times([fused_sequence], 3, 1)
                ms_2, _ = event_times([two_launch_sequence], 3, 1)
                ms_u, _ = event_times([unfused_sequence], 3, 1)
                others[lkey] = {
                    "workload": "LSTM, %d layers x %d steps, hidden %d, batch %d, gate matrix %dx%d %s, tiles %dx%d rank %d"
                                % (layers_, steps_, Hh, Bb, c.m, c.n, c.dtype, c.r, c.c, c.k),
                    "fused_sequence_ms": round(ms_f, 4), "fused_us_per_step": round(ms_f * 1e3 / (steps_ * layers_), 2),
                    "two_launch_sequence_ms": round(ms_2, 4), "two_launch_us_per_step": round(ms_2 * 1e3 / (steps_ * layers_), 2),
                    "unfused_sequence_ms": round(ms_u, 4),
                    "dense_equiv_tflops_fused": round(2.0 * c.m * c.n * Bb * steps_ * layers_ / (ms_f * 1e-3) / 1e12, 2)}
                del Wd, xs_, lws, xh, xh2, cs
            except Exception as e:
                others[lkey] = {"error": repr(e)}
        # backward pass through the masking layer: dX = (W o I_a)^T dY and dW = (dY X^T) o I_a
        for name in ("C2", "C3b", "paper_fc5_tiles"):
            key = "backward_" + name
            if wanted is not None and key not in wanted:
                continue
            try:
                c = workloads.CONFIGS.get(name) or general[name]
                d = workloads.make(c)
                de = lrbi.Desc(c.m, c.n, c.r, c.c, c.k)
                ip_, iz_ = factors_to_dev(de, d["Ip01"], d["Iz01"])
                Wl = rotated_weights(to_dev(d["W"], c.dtype))
                X_ = to_dev(d["X"], c.dtype)
                dY_ = torch.randn((c.m, c.N), device=dev, dtype=torch.float32).to(TD[c.dtype])
                dX_ = torch.empty((c.n, c.N), dtype=TD[c.dtype], device=dev)
                dWl = [torch.empty_like(Wi) for Wi in Wl]   # rotating outputs: every launch writes HBM-cold lines
                wb = lrbi.masked_gemm_t_workspace_bytes(de, DC[c.dtype], c.N)
                w_ = torch.empty(max(1, wb // 4), dtype=torch.float32, device=dev) if wb else None
                fns = [(lambda Wi=Wi: lrbi.masked_gemm_t(de, Wi, ip_, iz_, dY_, out=dX_, workspace=w_)) for Wi in Wl]
                ms_t, _ = event_times(fns, 6 * len(fns), len(fns))
                fns = [(lambda Gi=Gi: lrbi.masked_grad(de, dY_, X_, ip_, iz_, out=Gi)) for Gi in dWl]
                ms_g, _ = event_times(fns, 6 * len(fns), len(fns))
                fl = 2.0 * c.m * c.n * c.N
                byt_t = (c.m * c.n + c.m * c.N + c.n * c.N) * 2 + lrbi.index_bits(de)["lrbi_bits"] / 8
                others[key] = {
                    "N": c.N, "dtype": c.dtype,
                    "gemm_t_ms_cold": round(ms_t, 5), "gemm_t_tflops_dense_equiv": round(fl / (ms_t * 1e-3) / 1e12, 2),
                    "gemm_t_GBs": round(byt_t / (ms_t * 1e-3) / 1e9, 1),
                    "grad_ms": round(ms_g, 5), "grad_tflops_dense_equiv": round(fl / (ms_g * 1e-3) / 1e12, 2),
                    "grad_GBs": round(byt_t / (ms_g * 1e-3) / 1e9, 1),
                    "grad_hbm_frac": round(byt_t / (ms_g * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
                del Wl, dWl, X_, dY_, dX_
            except Exception as e:
                others[key] = {"error": repr(e)}
        # non-negative factorisation of |W| per tile (Algorithm 1's first step): multiplicative updates on C2 and C3
        for name in ("C2", "C3a", "C4", "paper_fc5_tiles"):
            key = "nmf_" + (name[:2] if name in workloads.CONFIGS else name)
            if wanted is not None and key not in wanted:
                continue
            try:
                c = workloads.CONFIGS.get(name) or general[name]
                d = workloads.make(c, want_x=False)
                de = lrbi.Desc(c.m, c.n, c.r, c.c, c.k)
                W_ = to_dev(d["W"], c.dtype)
                f = workloads.make_real_factors(c)
                Mp_, Mz_ = torch.from_numpy(f["Mp"]).to(dev) + 0.05, torch.from_numpy(f["Mz"]).to(dev) + 0.05
                nws = torch.empty(lrbi.nmf_workspace_bytes(de), dtype=torch.uint8, device=dev)
                iters_ = 20
                run = lambda: lrbi.nmf(de, W_, Mp_, Mz_, iters_, workspace=nws)
                run()
                torch.cuda.synchronize()
                ts = []
                for _ in range(3):
                    e0 = torch.cuda.Event(enable_timing=True)
                    e1 = torch.cuda.Event(enable_timing=True)
                    e0.record()
                    run()
                    e1.record()
                    torch.cuda.synchronize()
                    ts.append(e0.elapsed_time(e1))
                ms = float(sorted(ts)[1])
                fl = iters_ * 4.0 * c.m * c.n * c.k  # two products with the magnitude matrix per iteration
                others[key] = {"workload": "%s: |W| %dx%d %s, tiles %dx%d, rank %d, %d multiplicative updates"
                                           % (key[4:], c.m, c.n, c.dtype, c.r, c.c, c.k, iters_),
                               "ms": round(ms, 4), "us_per_iteration": round(ms * 1e3 / iters_, 2),
                               "tflops_fp32": round(fl / (ms * 1e-3) / 1e12, 2),
                               "alu_frac_of_157_tflops": round(fl / (ms * 1e-3) / 1e12 / 157.3, 4)}
                del W_, Mp_, Mz_, nws
            except Exception as e:
                others[key] = {"error": repr(e)}
        # the whole threshold search of Algorithm 1 for a layer: sort, then n_sp x steps candidates (W stays in the
        # last-level cache between candidates, as it would in real use); eager launches, HIP events around them
        if wanted is None or "alg1_search_C2" in wanted:
            try:
                c = workloads.CONFIGS["C2"]
                d = workloads.make(c, want_x=False)
                f = workloads.make_real_factors(c)
                de = lrbi.Desc(c.m, c.n, c.r, c.c, c.k)
                W_ = to_dev(d["W"], c.dtype)
                Mp_, Mz_ = torch.from_numpy(f["Mp"]).to(dev), torch.from_numpy(f["Mz"]).to(dev)
                sws = torch.empty(lrbi.search_workspace_bytes(de), dtype=torch.uint8, device=dev)
                S_, sweep, steps_, tol = 0.90, [0.86 + 0.0125 * i for i in range(8)], 10, int(0.005 * c.r * c.c)
                run = lambda: lrbi.search_thresholds(de, W_, f["w_threshold"], Mp_, Mz_, S_, sweep, steps_, tol,
                                                     want_factors=True, workspace=sws)
                run()
                torch.cuda.synchronize()
                ts = []
                for _ in range(5):
                    e0 = torch.cuda.Event(enable_timing=True)
                    e1 = torch.cuda.Event(enable_timing=True)
                    e0.record()
                    res_ = run()
                    e1.record()
                    torch.cuda.synchronize()
                    ts.append(e0.elapsed_time(e1))
                ms = float(sorted(ts)[2])
                ncand = len(sweep) * steps_
                eligible = int(((res_[2] - round((1 - S_) * c.r * c.c)).abs() <= tol).sum())
                others["alg1_search_C2"] = {
                    "workload": "C2: W %dx%d %s, U(0,1) factors, S = %.2f, %d S_p values x %d bisection steps, "
                                "tolerance %d ones" % (c.m, c.n, c.dtype, S_, len(sweep), steps_, tol),
                    "search_ms": round(ms, 4), "candidates": ncand, "ms_per_candidate": round(ms / ncand, 5),
                    "tile_candidates_per_s": round(c.tiles * ncand / (ms * 1e-3), 1),
                    "tiles_with_eligible_winner": eligible, "tiles": c.tiles}
                del W_, Mp_, Mz_, sws
            except Exception as e:
                others["alg1_search_C2"] = {"error": repr(e)}
        out["others"] = others

        # measured ceilings on this machine (context for the fractions above, not product code):
        # a plain 1 GiB fill, and the vendor library's dense GEMM of the same shape and dtype
        if wanted is None or "ceilings" in wanted:
            ceilings = {}
            try:
                buf = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
                ms, _ = event_times([lambda: buf.fill_(1)], 10, 3)
                ceilings["fill_1GiB_GBs"] = round((1 << 30) / (ms * 1e-3) / 1e9, 1)
                del buf
            except Exception as e:
                ceilings["fill_1GiB_GBs"] = {"error": repr(e)}
            try:  # a plain read: the framework's own sum over 1 GiB of fp32, three buffers in turn
                bufs = [torch.ones(1 << 28, dtype=torch.float32, device=dev) for _ in range(3)]
                for t in bufs:
                    t.sum()
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()  # eager launches (a library reduction is not captured into a graph here): 0.25 ms each
                for _ in range(3):
                    for t in bufs:
                        t.sum()
                e1.record()
                torch.cuda.synchronize()
                ceilings["sum_1GiB_GBs"] = round((1 << 30) / (e0.elapsed_time(e1) / 9 * 1e-3) / 1e9, 1)
                del bufs
            except Exception as e:
                ceilings["sum_1GiB_GBs"] = {"error": repr(e)}
            for name in ("C2", "C3b", "C5"):
                try:
                    c = workloads.CONFIGS[name]
                    A = torch.randn((c.m, c.n), device=dev, dtype=torch.float32).to(TD[c.dtype])
                    B = torch.randn((c.n, c.N), device=dev, dtype=torch.float32).to(TD[c.dtype])
                    C = torch.empty((c.m, c.N), device=dev, dtype=TD[c.dtype])
                    ms, _ = event_times([lambda: torch.matmul(A, B, out=C)], 20, 5)
                    ceilings["dense_matmul_" + name] = {
                        "avg_launch_ms": round(ms, 5),
                        "tflops": round(2.0 * c.m * c.n * c.N / (ms * 1e-3) / 1e12, 1),
                        "note": "torch.matmul (hipBLASLt), unmasked, same buffer every launch"}
                    del A, B, C
                except Exception as e:
                    ceilings["dense_matmul_" + name] = {"error": repr(e)}
            out["measured_ceilings"] = ceilings

    # ------------------------------------------------------------------ oracle on the host cores
    if not args.no_cpu:
        from oracle import lrbi_oracle as orc
        cores = max(1, min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "0")) or (os.cpu_count() or 1)))
        Wd = workloads.to_float64(data["W"], cfg.dtype)
        Xd = workloads.to_float64(data["X"], cfg.dtype)
        c0 = time.perf_counter()
        M = orc.decode_mask(data["Ip01"], data["Iz01"], cfg.m, cfg.n, cfg.r, cfg.c, cfg.k)
        c1 = time.perf_counter()
        orc.masked_gemm(Wd, M, Xd, threads=cores)
        c2 = time.perf_counter()
        out["cpu_baseline"] = {
            "value": round(flops / (c2 - c0) / 1e12, 5), "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": "the whole C2 step once: plain-C decode of the 4096x9216 mask (1 thread, %.2f s) + fp64 masked "
                      "product at N=128 (OpenMP over rows, %d threads, %.2f s)" % (c1 - c0, cores, c2 - c1),
            "decode_gbit_s": round(cfg.m * cfg.n / (c1 - c0) / 1e9, 4)}

    print(json.dumps(out))


if __name__ == "__main__":
    main()
