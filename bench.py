#!/usr/bin/env python3
"""Benchmark of the HDC hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

A step is one pass of the classical pipeline over the ISOLET-shaped synthetic workload
(D=10000, F=617, L=64, C=26, 6238 train / 1559 test samples, all resident in HBM):
    encode(train) -> classical accumulate -> majority binarise -> encode(test) -> Hamming search.
Prints ONE JSON line.  `value` = encoded+trained samples/s (N_train over the device time of
encode(train) + train + binarise, from events inside the timed steps); Hamming queries/s,
the online-training rate (UCIHAR-shaped config) and large-N figures for the HBM-bound
kernels ride along as extra keys.  `roofline` describes the dominant kernel (encode_kernel,
VALU-bound); `cpu_baseline` is the CPU oracle timed on this machine's host cores on a bounded
sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X figures used for the rooflines
HBM_PEAK_GBS = 8000.0
# Plain 32-bit VALU peak: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz = 39.3 T lane-ops/s
# (one v_bitop3_b32 / v_xor_b32 / v_bcnt per lane per clock; half the fp32 FMA-flop figure of
# 157.3 TFLOP/s, which counts 2 flops per FMA and the packed-fp32 dual issue).
VALU_PEAK_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12
MFMA_FP4_PEAK_TFLOPS = 10100.0    # MI355X published dense FP4 matrix peak
FP64_PEAK_TFLOPS = 78.6           # MI355X published fp64 vector peak (FMA = 2 flop)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true")
    ap.add_argument("--no-kernel-events", action="store_true",
                    help="diagnosis: do not bracket the hot kernels with events in the timed region (no roofline)")
    ap.add_argument("--copy-reference", action="store_true",
                    help="only run a 1 GiB device copy 10 times (known-size kernel that scales the "
                         "FETCH_SIZE / WRITE_SIZE counters) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "run it with --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2206_04746_amd import binding  # fails loudly if libhdc.so is missing
    from workloads import make_workload

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    K, Wm = max(1, args.steps), max(0, args.warmup)
    if args.copy_reference:
        a = torch.ones(1 << 28, dtype=torch.int32, device="cuda")
        b = torch.empty_like(a)
        for _ in range(10):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"copy_reference_bytes_read": a.numel() * 4, "copy_reference_bytes_written": a.numel() * 4,
                          "launches": 10}))
        return 0

    wl = make_workload(2)
    xt_h, yt_h = wl.train()
    xs_h, ys_h = wl.test()
    ntr, nte = xt_h.shape[0], xs_h.shape[0]
    ctx = binding.Context(wl.D, wl.F, wl.L, wl.C, wl.item, wl.level, wl.tie, wl.lo, wl.scale, wl.dtype)
    W = ctx.W
    dev = "cuda"
    xt, yt = torch.from_numpy(xt_h).to(dev), torch.from_numpy(yt_h).to(dev)
    xs = torch.from_numpy(xs_h).to(dev)
    hv_t = torch.empty((ntr, W), dtype=torch.int32, device=dev)
    hv_s = torch.empty((nte, W), dtype=torch.int32, device=dev)
    acc = torch.zeros((wl.C, wl.D), dtype=torch.int32, device=dev)
    cn = torch.zeros(wl.C, dtype=torch.int64, device=dev)
    cls = torch.empty((wl.C, W), dtype=torch.int32, device=dev)
    dist = torch.empty((nte, wl.C), dtype=torch.int32, device=dev)
    pred = torch.empty(nte, dtype=torch.int32, device=dev)

    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(K)]

    def step(e=None):
        if e:
            e[0].record()
        ctx.hdc_encode(xt, hv_t)
        acc.zero_()
        cn.zero_()
        ctx.hdc_train_classical(hv_t, yt, acc, cn)
        ctx.hdc_binarize_classical(acc, cn, cls)
        if e:
            e[1].record()
        ctx.hdc_encode(xs, hv_s)
        if e:
            e[2].record()
        ctx.hdc_search(hv_s, cls, pred, dist)
        if e:
            e[3].record()

    for _ in range(Wm):
        step()
    torch.cuda.synchronize()
    # ---- the timed region: exactly K steps, stage boundaries marked by four events per step
    t0 = time.perf_counter()
    for k in range(K):
        step(ev[k])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / K
    # ---- the same K steps once more with every hot kernel bracketed by its own pair of events on
    # the launch stream (hdc_profile_*): per-kernel durations for the roofline.  Kept out of the
    # region above because the extra events hold the stream up between kernels (about 20 % of a
    # step of this size); a kernel's own duration is the same in both passes and in
    # profiles/bench_cfg2_kernel_stats.txt.
    ctx.hdc_profile_enable(not args.no_kernel_events)
    for k in ("encode", "encode_contract", "quantize", "accumulate", "search"):
        ctx.hdc_profile_read(k)
    for k in range(K):
        step()
    torch.cuda.synchronize()
    prof = {k: ctx.hdc_profile_read(k) for k in ("encode", "encode_contract", "quantize", "accumulate", "search")}
    ctx.hdc_profile_enable(False)
    t_train = np.array([e[0].elapsed_time(e[1]) for e in ev])    # ms: encode(train)+train+binarise
    t_enc_s = np.array([e[1].elapsed_time(e[2]) for e in ev])    # ms: encode(test)
    t_search = np.array([e[2].elapsed_time(e[3]) for e in ev])   # ms: search
    value = ntr / (t_train.mean() * 1e-3)
    queries = nte / (t_search.mean() * 1e-3)
    accuracy = float((pred.cpu().numpy() == ys_h).mean())

    # ---- roofline of the dominant kernel -------------------------------------------------
    # hdc_encode has two forms.  From 1024 samples on (here: both sets) it runs as a contraction
    # over the features on the matrix cores, encode_contract_kernel: per sample and varying dimension
    # one dot product of two F-bit vectors, 2 * F flops, on FP4 operands - the dominant kernel of
    # the step, priced against the FP4 matrix peak.  Smaller calls take
    # encode_kernel on the vector unit: one bind XOR + one full adder (two 3-input bit ops) per
    # (sample, feature, 32-bit word) = 3 * F * Wk lane-ops per sample, Wk the words it bundles
    # (dimensions that no level vector changes are constants of the model and are not computed).
    enc_ms, enc_launches = prof["encode"]
    ct_ms, ct_launches = prof["encode_contract"]
    Wk = ctx.hdc_encoded_words()
    ops_per_sample = 3.0 * wl.F * Wk
    # which calls took which form shows in the launch counts (the library decides by the call's size)
    ct_samples = 0 if ct_launches == 0 else ntr if ct_launches == K else ntr + nte
    valu_samples = ntr + nte - ct_samples
    valu_achieved = ops_per_sample * valu_samples * K / (enc_ms * 1e-3) / 1e12 if enc_ms > 0 else 0.0
    valu_kernel = {
        "kernel": "encode_kernel", "bound": "alu", "achieved": round(valu_achieved, 3),
        "peak": round(VALU_PEAK_TOPS, 2), "unit": "Tlane-op/s", "frac": round(valu_achieved / VALU_PEAK_TOPS, 4),
        "avg_launch_us": round(enc_ms * 1e3 / max(1, enc_launches), 2), "launches": enc_launches,
        "samples_per_launch": valu_samples // max(1, enc_launches // K) if enc_launches else 0,
        "algorithmic_ops_per_sample": ops_per_sample, "words_bundled_of": [Wk, W],
    }
    if ct_launches:
        flops_per_sample = 2.0 * wl.F * Wk * 32
        achieved = flops_per_sample * ct_samples * K / (ct_ms * 1e-3) / 1e12
        roofline = {
            "kernel": "encode_contract_kernel", "bound": "mfma", "achieved": round(achieved, 2),
            "peak": MFMA_FP4_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / MFMA_FP4_PEAK_TFLOPS, 4),
            "traffic": _profiled_traffic("hdc::encode_contract_kernel"),
            "avg_launch_us": round(ct_ms * 1e3 / ct_launches, 2), "launches": ct_launches,
            "samples_per_step": ct_samples, "launches_per_step": ct_launches // K,
            "algorithmic_flops_per_sample": flops_per_sample,
            "dimensions_contracted_of": [Wk * 32, wl.D],
            "note": "quantise + contraction + bit placement in one kernel; the vector kernel it replaces took "
                    "83 us (6238 samples) and 33 us (1559) at 0.48 of the VALU peak over both",
        }
        if enc_launches:
            roofline["vector_kernel"] = valu_kernel
    else:
        roofline = dict(valu_kernel)
        roofline["traffic"] = _profiled_traffic("hdc::encode_kernel")
        roofline["frac_if_all_words_were_bundled"] = round(valu_achieved / VALU_PEAK_TOPS * W / max(1, Wk), 4)
    srch_ms, srch_launches = prof["search"]
    accu_ms, accu_launches = prof["accumulate"]
    kernels = {
        "search_kernel": {"avg_launch_us": round(srch_ms * 1e3 / max(1, srch_launches), 2),
                          "GBs": round((nte * W * 4 + nte * 4 * (wl.C + 1)) * srch_launches / (srch_ms * 1e-3) / 1e9, 2)
                          if srch_ms > 0 else 0.0},
        "accumulate_kernel": {"avg_launch_us": round(accu_ms * 1e3 / max(1, accu_launches), 2),
                              "GBs": round((ntr * W * 4 + ntr * 4) * accu_launches / (accu_ms * 1e-3) / 1e9, 2)
                              if accu_ms > 0 else 0.0},
        "quantize_kernel": {"avg_launch_us": round(prof["quantize"][0] * 1e3 / max(1, prof["quantize"][1]), 2)},
    }

    out = {
        "metric": "encoded+trained samples/sec and Hamming queries/sec at D=10000; % HBM roofline",
        "value": round(value, 1), "unit": "samples/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u32", "data": "synthetic",
        "config": {"workload": "configs[1]: classical HDC, D=10000, F=617 fp32, L=64, C=26, "
                               "6238 train / 1559 test (ISOLET shape, seeded Gaussian clusters)",
                   "step": "encode(train)+train_classical+binarize | encode(test) | search"},
        "queries_per_s": round(queries, 1),
        "encode_test_samples_per_s": round(nte / (t_enc_s.mean() * 1e-3), 1),
        "stage_ms": {"encode_train_plus_train": round(float(t_train.mean()), 4),
                     "encode_test": round(float(t_enc_s.mean()), 4),
                     "search": round(float(t_search.mean()), 4)},
        "test_accuracy": round(accuracy, 4),
        "roofline": roofline,
        "kernels": kernels,
    }

    if not args.no_extras:
        out["extras"] = extras(torch, binding, make_workload)
        # The same step recorded once in a HIP graph and replayed K times (one submission per step
        # instead of seven launches): what a serving loop would do.  Not `value`: reported beside it.
        try:
            pred_eager = pred.clone()
            side = torch.cuda.Stream()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                step()
            torch.cuda.synchronize()
            for _ in range(Wm):
                graph.replay()
            g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            g0.record()
            for _ in range(K):
                graph.replay()
            g1.record()
            torch.cuda.synchronize()
            out["extras"]["step_replayed_from_hip_graph"] = {
                "ms_per_step": round(g0.elapsed_time(g1) / K, 4), "steps": K,
                "same_predictions_as_eager": bool(torch.equal(pred, pred_eager))}
        except RuntimeError as err:   # the headline above does not depend on this
            out["extras"]["step_replayed_from_hip_graph"] = {"error": str(err)[:200]}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, xt_h, yt_h)
    ctx.close()
    print(json.dumps(out))
    return 0


def _profiled_traffic(kernel: str):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary (FETCH_SIZE and
    WRITE_SIZE in KiB per dispatch, scaled by the copy-kernel factors stated in that file); None
    if the summary is absent.  Counters cannot be collected from inside this process."""
    path = os.path.join(ROOT, "profiles", "encode_kernel_cfg2_pmc.txt")
    try:
        text = open(path).read()
    except OSError:
        return None
    import re
    scale = {"FETCH_SIZE": 2.0, "WRITE_SIZE": 1.0}
    m = re.search(r"FETCH_SIZE x ([0-9.]+), WRITE_SIZE x ([0-9.]+)", text)
    if m:
        scale = {"FETCH_SIZE": float(m.group(1)), "WRITE_SIZE": float(m.group(2))}
    total = 0.0
    for ctr in ("FETCH_SIZE", "WRITE_SIZE"):
        # one line per kernel instantiation: average over all launches of all of them
        rows = re.findall(re.escape(kernel) + r"[^\n]*," + ctr + r",launches=(\d+),mean=([0-9.]+)", text)
        if not rows:
            return None
        launches = sum(int(n) for n, _ in rows)
        total += sum(int(n) * float(m) for n, m in rows) / launches * 1024.0 * scale[ctr]
    return round(total, 1)


def _timed(torch, fn, reps):
    fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def extras(torch, binding, make_workload):
    """Large-N figures for the HBM-bound kernels (CHB-MIT-shaped: C=2, one 1M-window chunk of
    random packed hypervectors) and the online trainer on the UCIHAR-shaped config."""
    res = {}
    dev = "cuda"
    # --- config 5 shape: search and classical accumulation over 1M packed rows
    wl5 = make_workload(5)
    ctx = binding.Context(wl5.D, wl5.F, wl5.L, wl5.C, wl5.item, wl5.level, wl5.tie, wl5.lo, wl5.scale, wl5.dtype)
    N = 1 << 20
    g = torch.Generator(device=dev)
    g.manual_seed(0)
    hv = torch.randint(-2 ** 31, 2 ** 31 - 1, (N, ctx.W), dtype=torch.int32, device=dev, generator=g)
    hv[:, -1] &= (1 << (wl5.D - 32 * (ctx.W - 1))) - 1
    y = (torch.rand(N, device=dev, generator=g) < 0.01).to(torch.int32)
    cls = hv[:2].clone()
    pred = torch.empty(N, dtype=torch.int32, device=dev)
    acc = torch.zeros((2, wl5.D), dtype=torch.int32, device=dev)
    cn = torch.zeros(2, dtype=torch.int64, device=dev)
    bytes_rows = N * ctx.W * 4
    ms = _timed(torch, lambda: ctx.hdc_search(hv, cls, pred, None), 5)
    res["search_1M_C2"] = {"ms": round(ms, 4), "queries_per_s": round(N / ms * 1e3, 0),
                           "GBs": round((bytes_rows + 4 * N) / ms / 1e6, 1),
                           "frac_hbm": round((bytes_rows + 4 * N) / ms / 1e6 / HBM_PEAK_GBS, 4)}
    # the same stream against 26 class vectors (ISOLET's class count): from 9 classes on the search is
    # a dense contraction and runs on the matrix cores (4-bit float MFMA, 32 class slots x 32 queries
    # x 64 bits per instruction)
    ctx26 = binding.Context(wl5.D, wl5.F, wl5.L, 26, wl5.item, wl5.level, wl5.tie, wl5.lo, wl5.scale, wl5.dtype)
    cls26 = hv[:26].clone()
    ms = _timed(torch, lambda: ctx26.hdc_search(hv, cls26, pred, None), 5)
    res["search_1M_C26"] = {"ms": round(ms, 4), "queries_per_s": round(N / ms * 1e3, 0),
                            "GBs": round((bytes_rows + 4 * N) / ms / 1e6, 1),
                            "frac_hbm": round((bytes_rows + 4 * N) / ms / 1e6 / HBM_PEAK_GBS, 4),
                            "mfma_Pflops": round(2.0 * N * 32 * ctx.W * 32 / (ms * 1e-3) / 1e15, 3),
                            "frac_mfma_fp4": round(2.0 * N * 32 * ctx.W * 32 / (ms * 1e-3) / 1e15 / 10.1, 4)}
    ctx26.close()
    del cls26
    ms = _timed(torch, lambda: ctx.hdc_train_classical(hv, y, acc, cn), 5)
    res["train_classical_1M_C2"] = {"ms": round(ms, 4), "samples_per_s": round(N / ms * 1e3, 0),
                                    "GBs": round((bytes_rows + 4 * N) / ms / 1e6, 1),
                                    "frac_hbm": round((bytes_rows + 4 * N) / ms / 1e6 / HBM_PEAK_GBS, 4)}
    # the stand-alone primitives of Sec. IV-B on the same 1M rows (all HBM-bound streams)
    nbits = 1 << 17                     # the byte matrix is 8x the packed one: 128k rows = 1.3 GB
    bits = torch.empty((nbits, wl5.D), dtype=torch.uint8, device=dev)
    hsum = torch.empty(N, dtype=torch.int32, device=dev)
    vsum = torch.empty(wl5.D, dtype=torch.int32, device=dev)
    ms = _timed(torch, lambda: ctx.hdc_unpack(hv[:nbits], bits), 5)
    b = nbits * (ctx.W * 4 + wl5.D)
    res["unpack_128k"] = {"ms": round(ms, 4), "GBs": round(b / ms / 1e6, 1), "frac_hbm": round(b / ms / 1e6 / HBM_PEAK_GBS, 4)}
    hv5p = torch.empty((nbits, ctx.W), dtype=torch.int32, device=dev)
    ms = _timed(torch, lambda: ctx.hdc_pack(bits, hv5p), 5)
    res["pack_128k"] = {"ms": round(ms, 4), "GBs": round(b / ms / 1e6, 1), "frac_hbm": round(b / ms / 1e6 / HBM_PEAK_GBS, 4)}
    ms = _timed(torch, lambda: ctx.hdc_hsum(hv, hsum), 5)
    res["hsum_1M"] = {"ms": round(ms, 4), "GBs": round((bytes_rows + 4 * N) / ms / 1e6, 1),
                      "frac_hbm": round((bytes_rows + 4 * N) / ms / 1e6 / HBM_PEAK_GBS, 4)}
    ms = _timed(torch, lambda: ctx.hdc_vsum(hv, vsum), 5)
    res["vsum_1M"] = {"ms": round(ms, 4), "GBs": round(bytes_rows / ms / 1e6, 1),
                      "frac_hbm": round(bytes_rows / ms / 1e6 / HBM_PEAK_GBS, 4)}
    del bits, hv5p, hsum, vsum
    x5, _ = wl5.train(65536)
    x5d = torch.from_numpy(x5).to(dev)
    hv5 = torch.empty((65536, ctx.W), dtype=torch.int32, device=dev)
    ms = _timed(torch, lambda: ctx.hdc_encode(x5d, hv5), 3)
    res["encode_64k_cfg5"] = {"ms": round(ms, 4), "samples_per_s": round(65536 / ms * 1e3, 0),
                              "frac_mfma_fp4": round(2.0 * wl5.F * ctx.hdc_encoded_words() * 32 * 65536 / (ms * 1e-3)
                                                     / 1e12 / MFMA_FP4_PEAK_TFLOPS, 4),
                              "note": "whole hdc_encode (one contraction launch: quantise + bundle + placement), "
                                      "2 flops per (feature, varying dimension) against the FP4 matrix peak"}
    ctx.close()
    del hv, y, pred, x5d, hv5
    # --- config 3 shape (digit images, u8, L = 256, about 80 % of the pixels in bin 0): hdc_encode
    # (all features; for this model the contraction on the matrix cores, 14 MFMA steps per tile)
    # against the call that bundles only the features that leave bin 0 (same bits out)
    wl3 = make_workload(3)
    ctx = binding.Context(wl3.D, wl3.F, wl3.L, wl3.C, wl3.item, wl3.level, wl3.tie, wl3.lo, wl3.scale, wl3.dtype)
    x3, _ = wl3.train()
    x3d = torch.from_numpy(x3).to(dev)
    n3 = x3.shape[0]
    hv3 = torch.empty((n3, ctx.W), dtype=torch.int32, device=dev)
    ms_d = _timed(torch, lambda: ctx.hdc_encode(x3d, hv3), 3)
    ms_s = _timed(torch, lambda: ctx.hdc_encode_sparse(x3d, hv3), 3)
    res["encode_cfg3_dense_vs_sparse"] = {
        "samples": n3, "features_not_in_bin0": round(float((x3 != 0).mean()), 4),
        "dense_ms": round(ms_d, 4), "dense_samples_per_s": round(n3 / ms_d * 1e3, 0),
        "sparse_ms": round(ms_s, 4), "sparse_samples_per_s": round(n3 / ms_s * 1e3, 0),
        "speedup": round(ms_d / ms_s, 2)}
    ctx.close()
    del x3d, hv3
    # --- config 4 shape: online training, one epoch over 7352 samples (a dependency chain)
    wl4 = make_workload(4)
    ctx = binding.Context(wl4.D, wl4.F, wl4.L, wl4.C, wl4.item, wl4.level, wl4.tie, wl4.lo, wl4.scale, wl4.dtype)
    x4, y4 = wl4.train()
    x4d, y4d = torch.from_numpy(x4).to(dev), torch.from_numpy(y4).to(dev)
    hv4 = torch.empty((x4.shape[0], ctx.W), dtype=torch.int32, device=dev)
    ctx.hdc_encode(x4d, hv4)
    acc4 = torch.zeros((wl4.C, wl4.D), dtype=torch.float32, device=dev)

    def online():
        acc4.zero_()
        ctx.hdc_train_online(hv4, y4d, acc4, epochs=1, lr=wl4.lr)
    ms = _timed(torch, online, 2)
    res["train_online_cfg4_1epoch"] = {"ms": round(ms, 3), "us_per_step": round(ms * 1e3 / x4.shape[0], 3),
                                       "samples_per_s": round(x4.shape[0] / ms * 1e3, 0)}
    # --- batched online training over the same set: the paper's batch-size axis (Sec. VI-D2).
    # The two big kernels are fp64 FMA work on the vector unit: C*D per sample in the forward
    # step, cb*D in the backward step (cb = C rounded up to 2/4/8/16 coefficient slots).
    cb = next(w for w in (2, 4, 8, 16, wl4.C) if w >= wl4.C)
    sweep = {}
    for batch in (8, 64, 512, 2048, 8192):
        def batched(b=batch):
            acc4.zero_()
            ctx.hdc_train_online_batched(hv4, y4d, acc4, b, epochs=1, lr=wl4.lr)
        ms = _timed(torch, batched, 3)
        entry = {"ms": round(ms, 4), "samples_per_s": round(x4.shape[0] / ms * 1e3, 0),
                 "speedup_vs_batch1_chain": round(res["train_online_cfg4_1epoch"]["ms"] / ms, 1)}
        if batch >= 2048:
            ctx.hdc_profile_enable(True)
            batched()
            torch.cuda.synchronize()
            f_ms, f_n = ctx.hdc_profile_read("online_fwd")
            b_ms, b_n = ctx.hdc_profile_read("online_bwd")
            ctx.hdc_profile_enable(False)
            n = x4.shape[0]
            entry["fwd_us"] = round(f_ms * 1e3, 2)
            entry["bwd_us"] = round(b_ms * 1e3, 2)
            entry["fwd_frac_fp64_valu"] = round(2.0 * n * wl4.C * wl4.D / (f_ms * 1e-3) / 1e12 / FP64_PEAK_TFLOPS, 4)
            entry["bwd_frac_fp64_valu"] = round(2.0 * n * cb * wl4.D / (b_ms * 1e-3) / 1e12 / FP64_PEAK_TFLOPS, 4)
        sweep[str(batch)] = entry
    res["train_online_batched_cfg4_1epoch"] = sweep
    # cosine-similarity inference of the train set against the trained accumulators
    pred4 = torch.empty(x4.shape[0], dtype=torch.int32, device=dev)
    ms = _timed(torch, lambda: ctx.hdc_search_cosine(hv4, acc4, pred4, None), 5)
    res["search_cosine_cfg4"] = {"ms": round(ms, 4), "queries_per_s": round(x4.shape[0] / ms * 1e3, 0),
                                 "frac_fp64_valu": round(2.0 * x4.shape[0] * wl4.C * wl4.D / (ms * 1e-3) / 1e12
                                                         / FP64_PEAK_TFLOPS, 4)}
    ctx.close()
    del hv4, x4d
    # the same trainer with 26 classes (config 2 shape): beyond 16 classes the backward step
    # works from per-class lists of the samples that carry a non-zero weight
    wl2 = make_workload(2)
    ctx = binding.Context(wl2.D, wl2.F, wl2.L, wl2.C, wl2.item, wl2.level, wl2.tie, wl2.lo, wl2.scale, wl2.dtype)
    x2, y2 = wl2.train()
    x2d, y2d = torch.from_numpy(x2).to(dev), torch.from_numpy(y2).to(dev)
    hv2 = torch.empty((x2.shape[0], ctx.W), dtype=torch.int32, device=dev)
    ctx.hdc_encode(x2d, hv2)
    acc2 = torch.zeros((wl2.C, wl2.D), dtype=torch.float32, device=dev)

    def batched26():
        acc2.zero_()
        ctx.hdc_train_online_batched(hv2, y2d, acc2, 8192, epochs=1, lr=wl2.lr)
    ms = _timed(torch, batched26, 3)
    ctx.hdc_profile_enable(True)
    batched26()
    torch.cuda.synchronize()
    f_ms, _ = ctx.hdc_profile_read("online_fwd")
    b_ms, _ = ctx.hdc_profile_read("online_bwd")
    ctx.hdc_profile_enable(False)
    res["train_online_batched_cfg2_1epoch_batch8192"] = {
        "ms": round(ms, 4), "samples_per_s": round(x2.shape[0] / ms * 1e3, 0),
        "fwd_us": round(f_ms * 1e3, 2), "bwd_us": round(b_ms * 1e3, 2),
        "fwd_frac_fp64_valu": round(2.0 * x2.shape[0] * wl2.C * wl2.D / (f_ms * 1e-3) / 1e12 / FP64_PEAK_TFLOPS, 4)}
    ctx.close()
    del hv2, x2d, acc2

    # --- the whole classical step (as timed for `value`) along the paper's dimension axis
    # (Sec. VI-D1, ISOLET shape) and at the small-feature PAMAP shape of Table II
    def pipeline(wl, ntr, nte):
        c = binding.Context(wl.D, wl.F, wl.L, wl.C, wl.item, wl.level, wl.tie, wl.lo, wl.scale, wl.dtype)
        xt, yt = wl.train(ntr)
        xs, _ = wl.test(nte)
        xt, yt, xs = torch.from_numpy(xt).to(dev), torch.from_numpy(yt).to(dev), torch.from_numpy(xs).to(dev)
        ht = torch.empty((ntr, c.W), dtype=torch.int32, device=dev)
        hs = torch.empty((nte, c.W), dtype=torch.int32, device=dev)
        a = torch.zeros((wl.C, wl.D), dtype=torch.int32, device=dev)
        n = torch.zeros(wl.C, dtype=torch.int64, device=dev)
        m = torch.empty((wl.C, c.W), dtype=torch.int32, device=dev)
        p = torch.empty(nte, dtype=torch.int32, device=dev)

        def train():
            c.hdc_encode(xt, ht)
            a.zero_()
            n.zero_()
            c.hdc_train_classical(ht, yt, a, n)
            c.hdc_binarize_classical(a, n, m)

        def infer():
            c.hdc_encode(xs, hs)
            c.hdc_search(hs, m, p, None)
        t_ms, i_ms = _timed(torch, train, 20), _timed(torch, infer, 20)
        c.close()
        return {"train_ms": round(t_ms, 4), "train_samples_per_s": round(ntr / t_ms * 1e3, 0),
                "infer_ms": round(i_ms, 4), "queries_per_s": round(nte / i_ms * 1e3, 0)}
    res["dimension_sweep_isolet_shape"] = {
        str(D): pipeline(make_workload(2, D=D), 6238, 1559) for D in (1024, 2048, 4096, 8192, 16384, 32768)}
    wl6 = make_workload(6)
    res["pamap_shape"] = pipeline(wl6, wl6.n_train, wl6.n_test)
    return res


def cpu_baseline(wl, xt_h, yt_h):
    """The CPU oracle, as it stands, on a bounded prefix of the same train set (about 15 s)."""
    import oracle
    oracle.build()
    probe = 128
    t = time.perf_counter()
    oracle.encode(xt_h[:probe], wl.D, wl.L, wl.item, wl.level, wl.tie, wl.lo, wl.scale)
    per = (time.perf_counter() - t) / probe
    n = int(min(xt_h.shape[0], max(probe, 15.0 / max(per, 1e-9))))
    t = time.perf_counter()
    hv = oracle.encode(xt_h[:n], wl.D, wl.L, wl.item, wl.level, wl.tie, wl.lo, wl.scale)
    acc, cn = oracle.train_classical(hv, yt_h[:n], wl.D, wl.C)
    m = oracle.binarize_classical(acc, cn, wl.tie)
    dt = time.perf_counter() - t
    t = time.perf_counter()
    oracle.search(hv, m, wl.D)
    ds = time.perf_counter() - t
    return {"value": round(n / dt, 1), "unit": "samples/s", "cores": oracle.threads(), "kind": "oracle",
            "sample": f"first {n} of {xt_h.shape[0]} train samples of configs[1]: oracle encode + "
                      f"train_classical + binarize ({dt:.1f} s); search of the same {n} rows: "
                      f"{n / ds:.0f} queries/s",
            "queries_per_s": round(n / ds, 1)}


if __name__ == "__main__":
    sys.exit(main())
