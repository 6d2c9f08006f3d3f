#!/usr/bin/env python3
"""Benchmark of the HDC hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

The workload is the largest configuration that fits one GPU: the long-term-EEG-shaped stream
(D=10000, F=342 fp32 features, L=64 levels, C=2 classes, 5,000,000 windows with 1 % positives,
taken in five chunks of 1,000,000 windows; Sec. VI-E / Table II shape), all inputs resident in HBM.
A step is one pass of the whole path over it:
    for each chunk: encode -> classical accumulate;  majority binarise;  for each chunk: search.
Prints ONE JSON line.  `value` = encoded+trained windows/s (all windows over the device time of
the encode + train + binarise leg, median over the timed steps); `queries_per_s` comes from the
search leg.  `roofline` describes the dominant kernel (the contraction form of the encoder on a
1M-window chunk) against the FP4 matrix peak it runs on, with the HBM fraction of the same
launch next to it; `hbm_roofline` gives the HBM fractions of the two legs the metric names.
`cpu_baseline` is the CPU oracle timed on this machine's host cores (all cores and one thread) on a
bounded prefix of the same windows.  The smaller configurations ride along under `secondary`.
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
CHUNK_WINDOWS = 1_000_000         # the stream is taken in chunks of this many windows
PROFILE_STEPS = 40                # steps of the per-kernel timing pass (5 launches a step; 512 slots)


def _load_stream(torch, wl, n_windows, dev):
    """The first `n_windows` windows of the stream and their labels, generated block by block
    (independently seeded blocks of 65536 rows) on the host threads and copied to the GPU."""
    from concurrent.futures import ThreadPoolExecutor
    from workloads.synthetic import CHUNK as BLOCK
    x = torch.empty((n_windows, wl.F), dtype=torch.float32, device=dev)
    y = torch.empty(n_windows, dtype=torch.int32, device=dev)
    starts = list(range(0, n_windows, BLOCK))

    def make(s):
        return s, wl.train(min(BLOCK, n_windows - s), s)
    t0 = time.perf_counter()
    h2d = 0.0
    with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:
        for s, (xb, yb) in ex.map(make, starts):
            t = time.perf_counter()
            x[s:s + xb.shape[0]].copy_(torch.from_numpy(xb))
            y[s:s + yb.shape[0]].copy_(torch.from_numpy(yb))
            torch.cuda.synchronize()
            h2d += time.perf_counter() - t
    return x, y, time.perf_counter() - t0, h2d


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--windows", type=int, default=5_000_000,
                    help="windows of the stream (default: all 5,000,000 of the configuration)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true")
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

    dev = "cuda"
    wl = make_workload(5)
    N = int(args.windows)
    if not 0 < N <= wl.n_train:
        print("bench.py: --windows must be 1..5000000", file=sys.stderr)
        return 2
    x, y, gen_s, h2d_s = _load_stream(torch, wl, N, dev)
    ctx = binding.Context(wl.D, wl.F, wl.L, wl.C, wl.item, wl.level, wl.tie, wl.lo, wl.scale, wl.dtype)
    W = ctx.W
    chunks = [(s, min(N, s + CHUNK_WINDOWS)) for s in range(0, N, CHUNK_WINDOWS)]
    hv = torch.empty((N, W), dtype=torch.int32, device=dev)
    acc = torch.zeros((wl.C, wl.D), dtype=torch.int32, device=dev)
    cn = torch.zeros(wl.C, dtype=torch.int64, device=dev)
    cls = torch.empty((wl.C, W), dtype=torch.int32, device=dev)
    pred = torch.empty(N, dtype=torch.int32, device=dev)

    def step(e=None):
        if e:
            e[0].record()
        acc.zero_()
        cn.zero_()
        for a, b in chunks:
            ctx.hdc_encode(x[a:b], hv[a:b])
            ctx.hdc_train_classical(hv[a:b], y[a:b], acc, cn)
        ctx.hdc_binarize_classical(acc, cn, cls)
        if e:
            e[1].record()
        for a, b in chunks:
            ctx.hdc_search(hv[a:b], cls, pred[a:b], None)
        if e:
            e[2].record()

    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(K)]
    for _ in range(Wm):
        step()
    torch.cuda.synchronize()
    # ---- the timed region: exactly K steps, the two legs separated by events on the stream
    t0 = time.perf_counter()
    for k in range(K):
        step(ev[k])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / K
    t_train = np.array([e[0].elapsed_time(e[1]) for e in ev])    # ms: encode + train + binarise, all chunks
    t_search = np.array([e[1].elapsed_time(e[2]) for e in ev])   # ms: search, all chunks
    value = N / (float(np.median(t_train)) * 1e-3)
    queries = N / (float(np.median(t_search)) * 1e-3)
    # sanity of the trained model on the stream itself (the configuration searches what it trained on)
    y_h = y.cpu().numpy()
    p_h = pred.cpu().numpy()
    accuracy = float((p_h == y_h).mean())
    recall_pos = float((p_h[y_h == 1] == 1).mean()) if (y_h == 1).any() else None

    # ---- per-kernel durations: the same step again, every hot kernel bracketed by its own pair of
    # events on the launch stream (hdc_profile_*).  Kept out of the region above because the
    # extra events hold the stream up between kernels.  The work is counted from the launches
    # that were actually timed.
    kinds = ("encode", "encode_contract", "encode_wide", "quantize", "accumulate", "search")
    # (the chip idled while the predictions were checked on the host: the same warm-up as before the
    # timed region, or the first dozen launches run at a lower clock - seen in the kernel trace)
    for _ in range(Wm):
        step()
    torch.cuda.synchronize()
    ctx.hdc_profile_enable(True)
    for k in kinds:
        ctx.hdc_profile_read(k)
    psteps = min(K, PROFILE_STEPS)
    for _ in range(psteps):
        step()
    torch.cuda.synchronize()
    prof = {k: ctx.hdc_profile_read(k) for k in kinds}
    ctx.hdc_profile_enable(False)
    full = [b - a for a, b in chunks]
    per_launch = float(np.mean(full))                       # windows per launch (1,000,000 unless --windows cuts it)

    # Algorithmic work (Sec. III Eq. 1): per window and varying dimension one dot product of two
    # F-bit vectors = 2 F flops on the matrix cores (dimensions no level vector changes are
    # constants of the model); bytes: the features in, the packed row out.
    Wk = ctx.hdc_encoded_words()
    Dv = 32 * Wk
    enc_bytes = 4.0 * wl.F + 4.0 * W
    ct_ms, ct_n = prof["encode_wide"]
    ct_name = "encode_wide_kernel (quantise + contraction + bit placement, one launch per chunk, jobs of 128 windows)"
    if not ct_n:
        ct_ms, ct_n = prof["encode_contract"]
        ct_name = "encode_contract_kernel (quantise + contraction + bit placement, one launch per chunk)"
    en_ms, en_n = prof["encode"]
    if ct_n:
        assert ct_n == psteps * len(chunks), "timed launches of the encoder do not match the steps run"
        us = ct_ms * 1e3 / ct_n
        flops = 2.0 * wl.F * Dv * per_launch
        achieved = flops / (us * 1e-6) / 1e12
        gbs = enc_bytes * per_launch / (us * 1e-6) / 1e9
        roofline = {
            "kernel": ct_name,
            "bound": "mfma", "achieved": round(achieved, 1), "peak": MFMA_FP4_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": round(achieved / MFMA_FP4_PEAK_TFLOPS, 4),
            "traffic": None,
            "traffic_note": "HBM bytes per launch are in profiles/ (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this "
                            "command); counters cannot be read from inside the run",
            "avg_launch_us": round(us, 1), "launches": ct_n, "windows_per_launch": per_launch,
            "algorithmic_flops_per_window": 2.0 * wl.F * Dv, "dimensions_contracted_of": [Dv, wl.D],
            "hbm": {"algorithmic_bytes_per_window": enc_bytes, "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4)},
        }
    else:
        assert en_n, "no encoder launch was timed"
        us = en_ms * 1e3 / en_n
        ops = 3.0 * wl.F * Wk * (N * psteps / en_n)
        achieved = ops / (us * 1e-6) / 1e12
        roofline = {"kernel": "encode_kernel", "bound": "alu", "achieved": round(achieved, 3),
                    "peak": round(VALU_PEAK_TOPS, 2), "unit": "Tlane-op/s",
                    "frac": round(achieved / VALU_PEAK_TOPS, 4), "traffic": None,
                    "avg_launch_us": round(us, 1), "launches": en_n}
    ac_ms, ac_n = prof["accumulate"]
    se_ms, se_n = prof["search"]
    row_bytes = 4.0 * W + 4.0
    kernels = {}
    if ac_n:
        us = ac_ms * 1e3 / ac_n
        # (the kernel hdc_train_classical takes for long calls: rows of up to 320 words are streamed a
        # wave per row, without a grouping pass for up to four classes)
        acc_name = "accumulate_kernel" if W > 320 else ("accumulate_local_kernel" if wl.C <= 4 else "accumulate_rows_kernel")
        kernels[acc_name] = {"avg_launch_us": round(us, 1), "launches": ac_n,
                                        "frac_hbm": round(row_bytes * per_launch / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)}
    if se_n:
        us = se_ms * 1e3 / se_n
        kernels["search_rows16_kernel" if wl.C <= 8 else "search_mfma_kernel"] = {"avg_launch_us": round(us, 1), "launches": se_n,
                                    "frac_hbm": round(row_bytes * per_launch / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)}
    # HBM fractions of the two legs the metric names, from the step's own stage times: what the
    # method must move per window (features in, row out, row and label in again for training; row
    # in and prediction out for the search) over the leg's device time.
    train_bytes = enc_bytes + row_bytes
    hbm = {
        "encode_plus_train": {"algorithmic_bytes_per_window": train_bytes,
                              "frac": round(train_bytes * value / 1e9 / HBM_PEAK_GBS, 4)},
        "search": {"algorithmic_bytes_per_query": row_bytes,
                   "frac": round(row_bytes * queries / 1e9 / HBM_PEAK_GBS, 4)},
    }

    out = {
        "metric": "encoded+trained samples/sec and Hamming queries/sec at D=10000; % HBM roofline",
        "value": round(value, 1), "unit": "samples/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u32", "data": "synthetic",
        "config": {"workload": f"configs[4]: long-term-EEG-shaped classical HDC, D=10000, F=342 fp32, L=64, C=2, "
                               f"{N} windows (1 % positive, lognormal per channel) in {len(chunks)} chunks of "
                               f"{CHUNK_WINDOWS}",
                   "step": "per chunk: encode + train_classical; binarize; per chunk: search"},
        "queries_per_s": round(queries, 1),
        "stage_ms_median": {"encode_plus_train": round(float(np.median(t_train)), 4),
                            "search": round(float(np.median(t_search)), 4)},
        "stage_ms_mean": {"encode_plus_train": round(float(t_train.mean()), 4),
                          "search": round(float(t_search.mean()), 4)},
        "hbm_roofline": hbm,
        "accuracy_on_stream": round(accuracy, 4), "recall_of_positives": recall_pos,
        "roofline": roofline,
        "kernels": kernels,
        "input": {"generated_s": round(gen_s, 1), "h2d_s": round(h2d_s, 2),
                  "h2d_GBs": round((x.numel() * 4 + y.numel() * 4) / max(h2d_s, 1e-9) / 1e9, 2),
                  "note": "host-to-device copies are outside the timed region (the boundary takes device pointers)"},
    }
    ctx.close()
    del x, hv, pred
    torch.cuda.empty_cache()

    if not args.no_extras:
        out["secondary"] = secondary(torch, binding, make_workload, K)
        out["extras"] = extras(torch, binding, make_workload)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(out))
    return 0


def secondary(torch, binding, make_workload, K):
    """The small classical configuration (ISOLET shape: 6238 train / 1559 test samples, 26 classes)
    as one step of eight launches - bound by launch sizes, not by any roofline."""
    dev = "cuda"
    wl = make_workload(2)
    xt_h, yt_h = wl.train()
    xs_h, ys_h = wl.test()
    ntr, nte = xt_h.shape[0], xs_h.shape[0]
    ctx = binding.Context(wl.D, wl.F, wl.L, wl.C, wl.item, wl.level, wl.tie, wl.lo, wl.scale, wl.dtype)
    W = ctx.W
    xt, yt, xs = torch.from_numpy(xt_h).to(dev), torch.from_numpy(yt_h).to(dev), torch.from_numpy(xs_h).to(dev)
    hv_t = torch.empty((ntr, W), dtype=torch.int32, device=dev)
    hv_s = torch.empty((nte, W), dtype=torch.int32, device=dev)
    acc = torch.zeros((wl.C, wl.D), dtype=torch.int32, device=dev)
    cn = torch.zeros(wl.C, dtype=torch.int64, device=dev)
    cls = torch.empty((wl.C, W), dtype=torch.int32, device=dev)
    dist = torch.empty((nte, wl.C), dtype=torch.int32, device=dev)
    pred = torch.empty(nte, dtype=torch.int32, device=dev)
    K = max(K, 50)
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
    for _ in range(10):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(K):
        step(ev[k])
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / K
    t_train = float(np.median([e[0].elapsed_time(e[1]) for e in ev]))
    t_enc_s = float(np.median([e[1].elapsed_time(e[2]) for e in ev]))
    t_search = float(np.median([e[2].elapsed_time(e[3]) for e in ev]))
    res = {"workload": "configs[1]: D=10000, F=617 fp32, L=64, C=26, 6238 train / 1559 test",
           "steps": K, "ms_per_step": round(ms_per_step, 4),
           "encoded_plus_trained_samples_per_s": round(ntr / (t_train * 1e-3), 1),
           "queries_per_s": round(nte / (t_search * 1e-3), 1),
           "stage_ms_median": {"encode_train_plus_train": round(t_train, 4), "encode_test": round(t_enc_s, 4),
                               "search": round(t_search, 4)},
           "test_accuracy": round(float((pred.cpu().numpy() == ys_h).mean()), 4)}
    # The same step recorded once in a HIP graph and replayed (one submission per step).
    try:
        pred_eager = pred.clone()
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
        torch.cuda.synchronize()
        for _ in range(10):
            graph.replay()
        g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        g0.record()
        for _ in range(K):
            graph.replay()
        g1.record()
        torch.cuda.synchronize()
        res["step_replayed_from_hip_graph"] = {"ms_per_step": round(g0.elapsed_time(g1) / K, 4),
                                               "same_predictions_as_eager": bool(torch.equal(pred, pred_eager))}
    except RuntimeError as err:
        res["step_replayed_from_hip_graph"] = {"error": str(err)[:200]}
    ctx.close()
    return {"cfg2_step": res}


def _timed(torch, fn, reps):
    """Median device time of a call in ms: two untimed calls, then at least ten calls each between its own pair of events."""
    for _ in range(2):
        fn()
    torch.cuda.synchronize()
    reps = max(reps, 10)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in ev:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    return float(np.median([a.elapsed_time(b) for a, b in ev]))


def extras(torch, binding, make_workload):
    """Large-N figures for the HBM-bound kernels (CHB-MIT-shaped: C=2, one 1M-window chunk of
    random packed hypervectors) and the online trainer on the UCIHAR-shaped config."""
    res = {}
    dev = "cuda"
    # --- config 5 shape: search and classical accumulation over 1M packed rows
    wl5 = make_workload(5)
    ctx = binding.Context(wl5.D, wl5.F, wl5.L, wl5.C, wl5.item, wl5.level, wl5.tie, wl5.lo, wl5.scale, wl5.dtype)
    N = 1_000_000                       # the stream's chunk of windows
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
                            "mfma_Pflops": round(2.0 * N * 26 * wl5.D / (ms * 1e-3) / 1e15, 3),
                            "frac_mfma_fp4": round(2.0 * N * 26 * wl5.D / (ms * 1e-3) / 1e15 / 10.1, 4),
                            "note": "flops are the method's own 2 N C D (26 classes, 10000 dimensions)"}
    ctx26.close()
    del cls26
    # 124 classes: four passes over the class slots in one launch, the rows read once
    ctxm = binding.Context(wl5.D, wl5.F, wl5.L, 124, wl5.item, wl5.level, wl5.tie, wl5.lo, wl5.scale, wl5.dtype)
    clsm = hv[:124].clone()
    ms = _timed(torch, lambda: ctxm.hdc_search(hv, clsm, pred, None), 5)
    res["search_1M_C124"] = {"ms": round(ms, 4), "queries_per_s": round(N / ms * 1e3, 0),
                             "frac_hbm": round((bytes_rows + 4 * N) / ms / 1e6 / HBM_PEAK_GBS, 4),
                             "mfma_Pflops": round(2.0 * N * 124 * wl5.D / (ms * 1e-3) / 1e15, 3),
                             "frac_mfma_fp4": round(2.0 * N * 124 * wl5.D / (ms * 1e-3) / 1e15 / 10.1, 4)}
    ctxm.close()
    del clsm
    # D = 32768, 26 classes: a tile of 32 queries per block at a time (the rows are 4 KB each)
    wlL = make_workload(1, D=32768, C=26, F=3, L=2)
    ctxL = binding.Context(wlL.D, wlL.F, wlL.L, 26, wlL.item, wlL.level, wlL.tie, wlL.lo, wlL.scale, wlL.dtype)
    NL = 250_000
    hvL = hv.view(-1)[:NL * ctxL.W].view(NL, ctxL.W)
    clsL = hvL[:26].clone()
    ms = _timed(torch, lambda: ctxL.hdc_search(hvL, clsL, pred[:NL], None), 5)
    res["search_250k_D32768_C26"] = {"ms": round(ms, 4), "queries_per_s": round(NL / ms * 1e3, 0),
                                     "frac_hbm": round((NL * ctxL.W * 4 + 4 * NL) / ms / 1e6 / HBM_PEAK_GBS, 4),
                                     "frac_mfma_fp4": round(2.0 * NL * 26 * 32768 / (ms * 1e-3) / 1e15 / 10.1, 4)}
    ctxL.close()
    del clsL, hvL
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
    # --- config 2 shape at 65536 samples: the contraction encoder on a level table of Sec. III's
    # construction, and the vector kernel on a level table without any structure (random bits:
    # every dimension flips many times, nothing is level-invariant), the general case of Eq. (1)
    wl2 = make_workload(2)
    x2, _ = wl2.train(6238)
    x2 = np.ascontiguousarray(np.tile(x2, (11, 1))[:65536])
    x2d = torch.from_numpy(x2).to(dev)
    ctx = binding.Context(wl2.D, wl2.F, wl2.L, wl2.C, wl2.item, wl2.level, wl2.tie, wl2.lo, wl2.scale, wl2.dtype)
    hv2 = torch.empty((65536, ctx.W), dtype=torch.int32, device=dev)
    ms = _timed(torch, lambda: ctx.hdc_encode(x2d, hv2), 3)
    b2 = 4.0 * wl2.F + 4.0 * ctx.W
    res["encode_64k_cfg2"] = {"ms": round(ms, 4), "samples_per_s": round(65536 / ms * 1e3, 0),
                              "frac_mfma_fp4": round(2.0 * wl2.F * ctx.hdc_encoded_words() * 32 * 65536 / (ms * 1e-3)
                                                     / 1e12 / MFMA_FP4_PEAK_TFLOPS, 4),
                              "frac_hbm": round(b2 * 65536 / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    ctx.close()
    rng = np.random.default_rng(7)
    level_rand = rng.integers(0, 2 ** 32, size=wl2.level.shape, dtype=np.uint64).astype(np.uint32)
    level_rand[:, -1] &= np.uint32((1 << (wl2.D - 32 * (level_rand.shape[1] - 1))) - 1)
    ctx = binding.Context(wl2.D, wl2.F, wl2.L, wl2.C, wl2.item, level_rand, wl2.tie, wl2.lo, wl2.scale, wl2.dtype)
    ctx.hdc_profile_enable(True)
    ms = _timed(torch, lambda: ctx.hdc_encode(x2d, hv2), 3)
    k_ms, k_n = ctx.hdc_profile_read("encode")
    ctx.hdc_profile_enable(False)
    ops = 3.0 * wl2.F * ctx.hdc_encoded_words() * 65536
    res["encode_generic_64k"] = {
        "ms": round(ms, 4), "samples_per_s": round(65536 / ms * 1e3, 0),
        "encode_kernel_us": round(k_ms * 1e3 / max(1, k_n), 1),
        "frac_valu": round(ops / (k_ms * 1e-3 / max(1, k_n)) / 1e12 / VALU_PEAK_TOPS, 4) if k_n else None,
        "words_bundled_of": [ctx.hdc_encoded_words(), ctx.W],
        "note": "random level table (no structure): quantize_kernel + encode_kernel on the vector unit, "
                "3 lane-ops per (feature, word) against 39.3 T lane-ops/s"}
    ctx.close()
    # level vectors on a circle (what flips at level l flips back at level l + L/2: half of the
    # dimensions flip twice): the contraction follows such dimensions through two tiles of opposite sign
    half = wl2.L // 2
    first = rng.integers(1, half + 1, wl2.D)
    vary = rng.random(wl2.D) < 0.5
    change = np.zeros((wl2.L, wl2.D), dtype=np.uint8)
    dims = np.nonzero(vary)[0]
    change[first[dims], dims] = 1
    back = dims[first[dims] + half < wl2.L]
    change[first[back] + half, back] = 1
    bits = (rng.integers(0, 2, wl2.D, dtype=np.uint8)[None, :] ^ (np.cumsum(change, axis=0) & 1)).astype(np.uint8)
    padded = np.zeros((wl2.L, level_rand.shape[1] * 32), dtype=np.uint8)
    padded[:, :wl2.D] = bits
    level_circle = np.packbits(padded.reshape(wl2.L, -1, 32), axis=2, bitorder="little").view(np.uint32).reshape(wl2.L, -1)
    ctx = binding.Context(wl2.D, wl2.F, wl2.L, wl2.C, wl2.item, level_circle, wl2.tie, wl2.lo, wl2.scale, wl2.dtype)
    ctx.hdc_profile_enable(True)
    ms = _timed(torch, lambda: ctx.hdc_encode(x2d, hv2), 3)
    k_ms, k_n = ctx.hdc_profile_read("encode_contract")
    ctx.hdc_profile_enable(False)
    res["encode_circular_levels_64k"] = {
        "ms": round(ms, 4), "samples_per_s": round(65536 / ms * 1e3, 0),
        "contraction_kernel_us": round(k_ms * 1e3 / max(1, k_n), 1) if k_n else None,
        "dimensions_that_flip_twice": int(back.size),
        "note": "config-2 shape with circular level vectors: encode_contract_kernel, two tiles of opposite "
                "sign per 32 such dimensions; the vector kernel takes 0.98 ms on this table"}
    ctx.close()
    del x2d, hv2
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
    # the same input on a level table without structure (random level vectors: every dimension flips
    # many times, so hdc_encode runs the vector kernel on all 313 words): where the sparse call is meant for
    rng3 = np.random.default_rng(11)
    level3 = rng3.integers(0, 2 ** 32, size=wl3.level.shape, dtype=np.uint64).astype(np.uint32)
    level3[:, -1] &= np.uint32((1 << (wl3.D - 32 * (level3.shape[1] - 1))) - 1)
    ctx = binding.Context(wl3.D, wl3.F, wl3.L, wl3.C, wl3.item, level3, wl3.tie, wl3.lo, wl3.scale, wl3.dtype)
    ms_d = _timed(torch, lambda: ctx.hdc_encode(x3d, hv3), 3)
    ms_s = _timed(torch, lambda: ctx.hdc_encode_sparse(x3d, hv3), 3)
    res["encode_cfg3_random_levels_dense_vs_sparse"] = {
        "samples": n3, "dense_ms": round(ms_d, 4), "dense_samples_per_s": round(n3 / ms_d * 1e3, 0),
        "sparse_ms": round(ms_s, 4), "sparse_samples_per_s": round(n3 / ms_s * 1e3, 0),
        "speedup": round(ms_d / ms_s, 2),
        "note": "level vectors without structure: no contraction, no level-invariant dimensions; "
                "hdc_encode = quantize_kernel + encode_kernel over all words"}
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


def _omp_threads(n: int) -> None:
    """Sets the thread count of the OpenMP runtime the oracle's library uses (the oracle itself is
    left as it stands)."""
    import ctypes
    ctypes.CDLL("libgomp.so.1").omp_set_num_threads(int(n))


def cpu_baseline(wl):
    """The CPU oracle, as it stands, on a bounded prefix of the same stream: encode + classical
    training + binarise, then the search of the same windows; on all host cores (about 15 s) and
    on one thread (about 8 s)."""
    import oracle
    oracle.build()
    cores = oracle.threads()

    def run(n):
        x, y = wl.train(n)
        t = time.perf_counter()
        hv = oracle.encode(x, wl.D, wl.L, wl.item, wl.level, wl.tie, wl.lo, wl.scale)
        acc, cn = oracle.train_classical(hv, y, wl.D, wl.C)
        m = oracle.binarize_classical(acc, cn, wl.tie)
        dt = time.perf_counter() - t
        t = time.perf_counter()
        oracle.search(hv, m, wl.D)
        return dt, time.perf_counter() - t
    probe = 256
    per = run(probe)[0] / probe
    n_all = int(min(65536, max(probe, 15.0 / max(per, 1e-9))))
    dt, ds = run(n_all)
    _omp_threads(1)
    try:
        n_one = int(min(n_all, max(64, 8.0 / max(per * cores, 1e-9))))
        dt1, ds1 = run(n_one)
    finally:
        _omp_threads(cores)
    return {"value": round(n_all / dt, 1), "unit": "samples/s", "cores": cores, "kind": "oracle",
            "sample": f"first {n_all} of the 5,000,000 windows of configs[4]: oracle encode + train_classical + "
                      f"binarize ({dt:.1f} s); search of the same windows: {n_all / ds:.0f} queries/s",
            "queries_per_s": round(n_all / ds, 1),
            "one_thread": {"value": round(n_one / dt1, 1), "queries_per_s": round(n_one / ds1, 1),
                           "sample": f"first {n_one} windows, OpenMP limited to 1 thread ({dt1:.1f} s)"}}


if __name__ == "__main__":
    sys.exit(main())
