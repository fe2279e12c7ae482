#!/usr/bin/env python3
"""Benchmark of the Bi-Mask per-layer hot path on one MI355X.

One "step" is one pass of the whole path over one batch of synthetic input (Alg. 1 of the
paper, search included), per weight matrix: forward mask + compression, forward sparse GEMM,
K-candidate permutation search, backward mask + transposed compression, backward sparse GEMM.
Default workload: configuration 5, the largest -- the MLP block W_up 11008x4096 and
W_down 4096x11008, 8192 tokens, bf16, 2:4, K = 100; one step runs the path over both
matrices.  The ResNet-50 layer3 3x3 convolution (configuration 2, HBM-bound) is measured
with the same protocol in the same run and reported under "secondary".

Prints ONE JSON line.  All inputs are resident in HBM before the timed region; the
activation / gradient / output buffers rotate over several copies so that successive
steps do not find them in the 256 MB last-level cache.
"""
from __future__ import annotations

import argparse
import numpy as np
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

EVENT_EVERY = 4                # the dominant stage is bracketed by HIP events in one step out of this many
HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0 # MI355X published dense bf16 matrix peak


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=None,
                    help="workload configuration; default 5 (the largest) for the headline line, 2 for the diagnostics")
    ap.add_argument("--layer", type=int, default=-1,
                    help="layer index inside the configuration; -1 = every matrix of configs 1, 2, 5 in one step, layer 0 of configs 3, 4")
    ap.add_argument("--no-secondary", action="store_true", help="skip the config-2 figures that accompany the config-5 line")
    ap.add_argument("--no-context", action="store_true",
                    help="skip the dense library GEMMs (torch.matmul) timed beside the step for context")
    ap.add_argument("--copies", type=int, default=0, help="rotating buffer copies (0 = enough for 1 GiB)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--breakdown-reps", type=int, default=30)
    ap.add_argument("--all-layers", action="store_true",
                    help="network aggregate: time every layer of the configuration and print per-stage totals")
    ap.add_argument("--grouped", action="store_true",
                    help="mask and search steps of ALL layers of the configuration through the grouped entry points")
    ap.add_argument("--network-step", action="store_true",
                    help="one Bi-Mask step over ALL layers of the configuration end to end: grouped masks and searches, "
                         "one GEMM call per layer and direction")
    ap.add_argument("--gradient-gap", action="store_true",
                    help="diagnostic: relative gap between the approximate input gradient of Eq. (10) and the exact one of "
                         "Eq. (5), identity vs best-of-K permutation, K = 10, 100, 1000")
    ap.add_argument("--refine", action="store_true",
                    help="diagnostic: hill-climbing refinement of the search's winner by random exchange proposals "
                         "(time, eligible-block share, gradient gap)")
    ap.add_argument("--refine-network", action="store_true",
                    help="refinement of every layer's permutation: one call per layer against the grouped call")
    ap.add_argument("--search-table", action="store_true",
                    help="permutation search over all ResNet-50 layers for 2:4, 4:8, 1:4, 2:8, 1:16 (the shape of the paper's Table 6)")
    ap.add_argument("--only-stage", default=None,
                    help="diagnostic: repeat ONE stage of the step (forward_mask_compress, perm_search, backward_mask_compress, "
                         "sparse_gemm_fwd, sparse_gemm_bwd) back to back, `steps` times per matrix: its stand-alone time")
    ap.add_argument("--delta-t", type=int, default=100,
                    help="steps between two permutation searches (Sec. 4.1) for the amortised secondary figure")
    return ap.parse_args()


class LayerRun:
    """Device buffers of one layer and the calls of one step (no allocation per step)."""

    def __init__(self, layer, data, copies):
        import torch
        import paper_2302_06058_amd as bm
        from helpers import to_dev, i32_dev
        self.bm, self.layer, self.torch = bm, layer, torch
        L = layer
        self.dt = bm.BF16 if L.dtype == "bf16" else bm.F32
        tdt = torch.bfloat16 if L.dtype == "bf16" else torch.float32
        self.W = to_dev(data.W, L.dtype)
        self.perms = i32_dev(data.perms)
        X0, dY0 = to_dev(data.X, L.dtype), to_dev(data.dY, L.dtype)
        self.X = [X0] + [X0.clone() for _ in range(copies - 1)]
        self.dY = [dY0] + [dY0.clone() for _ in range(copies - 1)]
        dev = self.W.device
        self.Y = [torch.empty((L.T, L.I), dtype=tdt, device=dev) for _ in range(copies)]
        self.dX = [torch.empty((L.T, L.J), dtype=tdt, device=dev) for _ in range(copies)]
        s24 = L.N <= 2                         # operands in the sparse matrix instruction's 2-of-4 format
        wj, wi = bm.mask_words(L.J), bm.mask_words(L.I)
        self.B = torch.empty((L.I, wj), dtype=torch.int32, device=dev)
        self.Bbar = torch.empty((L.I, wj), dtype=torch.int32, device=dev)
        self.vf = torch.empty((bm.operand_elems(L.I, L.J, L.N, L.M),), dtype=tdt, device=dev)
        self.xf = torch.empty((bm.operand_index_words(L.I, L.J, L.N, L.M),), dtype=torch.int32, device=dev) if s24 else None
        self.vb = torch.empty((bm.operand_elems(L.J, L.I, L.N, L.M),), dtype=tdt, device=dev)
        self.xb = torch.empty((bm.operand_index_words(L.J, L.I, L.N, L.M),), dtype=torch.int32, device=dev) if s24 else None
        self.scores = torch.empty((L.K,), dtype=torch.int32, device=dev)
        self.best = torch.empty((1,), dtype=torch.int32, device=dev)
        self.P = torch.empty((L.I,), dtype=torch.int32, device=dev)
        self.ws_perm = torch.empty((max(16, bm.workspace_bytes(bm.WS_PERM_SEARCH, L.I, L.J, 0, L.K, self.dt, L.N, L.M)),),
                                   dtype=torch.uint8, device=dev)
        self.ws_bwd = torch.empty((max(16, bm.workspace_bytes(bm.WS_GEMM_BWD, L.I, L.J, L.T, 0, self.dt, L.N, L.M)),),
                                  dtype=torch.uint8, device=dev)
        self.copies = copies
        # every call of the step bound once to its marshalled arguments (one per rotating copy)
        st = torch.cuda.current_stream().cuda_stream
        N, M, I, J, T, K = L.N, L.M, L.I, L.J, L.T, L.K
        nbytes = lambda t: t.numel() * t.element_size()
        self.c_fwd_mask = bm.prepare("bimask_forward_mask_compress", self.W, I, J, J, self.dt, N, M, self.B,
                                     self.vf, self.xf, st)
        self.c_perm = bm.prepare("bimask_perm_search", self.B, I, J, N, M, self.perms, K, self.scores, self.best,
                                 self.P, self.ws_perm, nbytes(self.ws_perm), st)
        self.c_bwd_mask = bm.prepare("bimask_backward_mask_compress", self.W, I, J, J, self.dt, N, M, self.B, self.P,
                                     self.Bbar, self.vb, self.xb, st)
        self.c_gemm_fwd = [bm.prepare("bimask_sparse_gemm_fwd", self.X[r], T, J, self.vf, self.xf, I, J, self.dt, N, M,
                                      self.Y[r], I, None, 0, st) for r in range(copies)]
        self.c_gemm_bwd = [bm.prepare("bimask_sparse_gemm_bwd", self.dY[r], T, I, self.P, self.vb, self.xb, I, J,
                                      self.dt, N, M, self.dX[r], J, self.ws_bwd, nbytes(self.ws_bwd), st)
                           for r in range(copies)]
        # Order of one step: the three weight-side stages first, then the two GEMMs.  Alg. 1 lists the forward
        # GEMM before the search and the backward mask, but those two depend on W and B only, not on the forward
        # output, so they may run right after the forward mask -- while W and B are still in the last-level
        # cache instead of behind the GEMM's output.
        self.stages = [
            ("forward_mask_compress", self.s_fwd_mask),
            ("perm_search", self.s_perm),
            ("backward_mask_compress", self.s_bwd_mask),
            ("sparse_gemm_fwd", self.s_gemm_fwd),
            ("sparse_gemm_bwd", self.s_gemm_bwd),
        ]

    def s_fwd_mask(self, r):
        self.c_fwd_mask()

    def s_gemm_fwd(self, r):
        self.c_gemm_fwd[r]()

    def s_perm(self, r):
        self.c_perm()

    def s_bwd_mask(self, r):
        self.c_bwd_mask()

    def s_gemm_bwd(self, r):
        self.c_gemm_bwd[r]()

    def step(self, i):
        r = i % self.copies
        for _, fn in self.stages:
            fn(r)


def algorithmic(layer):
    """Algorithmic bytes / flops per call of each stage (what the method itself must move)."""
    L = layer
    e = 2 if L.dtype == "bf16" else 4
    s24 = L.N <= 2
    wbytes = L.I * L.J * ((e / 2 + 1 / 8) if s24 else e)       # 2-of-4 compressed (or dense masked) operand
    mask = L.I * L.J / 8
    return {
        "forward_mask_compress": {"bytes": L.I * L.J * e + mask + wbytes, "flops": 0},
        "sparse_gemm_fwd": {"bytes": e * L.T * L.J + e * L.T * L.I + wbytes, "flops": 2 * L.T * L.I * L.J},
        "perm_search": {"bytes": mask + 4 * L.K * L.I + 4 * L.K, "flops": 0},
        "backward_mask_compress": {"bytes": L.I * L.J * e + mask + mask + wbytes, "flops": 0},
        "sparse_gemm_bwd": {"bytes": e * L.T * L.I + e * L.T * L.J + wbytes, "flops": 2 * L.T * L.I * L.J},
    }


def _best(fn, reps=3, budget_s=2.5):
    """Best of up to `reps` timings of fn() in milliseconds (fewer when one run exceeds the budget)."""
    best = None
    for _ in range(reps):
        t0 = time.perf_counter()
        fn()
        dt = time.perf_counter() - t0
        best = dt if best is None else min(best, dt)
        if dt > budget_s:
            break
    return best * 1e3


def cpu_baseline(layers, datas):
    """The oracle as it stands on this machine's host cores, step by step (a reported baseline, not a target).

    Per matrix of the step: forward mask, candidate scores + arg-max, backward mask, the two compressions
    (the oracle's C loops: once on one thread, once with the same C functions called on row / candidate /
    row-block slices from `cores` threads) and the two float64 GEMMs (library matmul on `cores` threads),
    each the best of up to three runs.  Steps whose full size would take minutes are timed on a stated
    sample and scaled linearly to the full step."""
    import numpy as np
    from concurrent.futures import ThreadPoolExecutor
    import oracle
    from paper_2302_06058_amd import synth
    cores = max(1, min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "0") or 0) or (os.cpu_count() or 1)))
    pool = ThreadPoolExecutor(max_workers=cores)

    def par(fn, pieces):
        list(pool.map(fn, pieces))

    def chunks(n, unit, parts):
        per = -(-(n // unit) // parts) * unit
        return [(a, min(n, a + per)) for a in range(0, n, per)]

    t1 = {}
    tall = {}
    samples = []
    for L, d in zip(layers, datas):
        N, M, I, J, T, K = L.N, L.M, L.I, L.J, L.T, L.K
        W = synth.to_f64(d.W, L.dtype)
        add = lambda dct, k, v: dct.__setitem__(k, dct.get(k, 0.0) + v)
        # O1 forward mask (row groups are independent: slices of rows)
        B = oracle.forward_mask(W, N, M)
        add(t1, "forward_mask", _best(lambda: oracle.forward_mask(W, N, M)))
        rows = chunks(I, 1, cores)
        add(tall, "forward_mask", _best(lambda: par(lambda ab: oracle.forward_mask(W[ab[0]:ab[1]], N, M), rows)))
        # O2 + O3 scores of a candidate sample, scaled to K (candidates are independent)
        ks = min(K, 4 if float(I) * J > 4e6 else K)
        add(t1, "perm_search", _best(lambda: oracle.argmax_first(oracle.perm_scores(B, d.perms[:ks], N, M))) * K / ks)
        ka = min(K, max(ks, cores))
        add(tall, "perm_search", _best(lambda: par(lambda c: oracle.perm_scores(B, d.perms[c:c + 1], N, M), range(ka))) * K / ka)
        if ks < K:
            samples.append(f"{L.name}: scores of {ks} (1 thread) / {ka} ({cores} threads) of the {K} candidates, scaled")
        P = d.perms[0]
        # O4 backward mask (blocks of M permuted rows are independent: slices of the permutation)
        add(t1, "backward_mask", _best(lambda: oracle.backward_mask(W, B, P, N, M)))
        blks = chunks(I, M, cores)

        def bwd_slice(ab):
            # permuted rows a .. b-1: the same C function on that part of P (rows are read through P)
            Bb = np.empty((ab[1] - ab[0], J), dtype=np.uint8)
            sel = np.empty_like(Bb)
            import ctypes
            oracle._load().oracle_backward_mask(oracle._p(W), oracle._p(B), ctypes.c_int64(ab[1] - ab[0]), ctypes.c_int64(J), N, M,
                                                oracle._p(np.ascontiguousarray(P[ab[0]:ab[1]])), oracle._p(Bb), oracle._p(sel))
        add(tall, "backward_mask", _best(lambda: par(bwd_slice, blks)))
        # O5 the two compressions
        add(t1, "compress", _best(lambda: oracle.compress_fwd(W, B, N, M)) + _best(lambda: oracle.compress_bwd(W, B, P, N, M)))
        add(tall, "compress", _best(lambda: par(lambda ab: oracle.compress_fwd(W[ab[0]:ab[1]], B[ab[0]:ab[1]], N, M), rows)) * 2)
        # O6 float64 GEMMs on a token sample, all cores (library matmul)
        ts = min(T, max(64, int(2e11 / (2.0 * I * J))))
        X, dY = synth.to_f64(d.X[:ts], L.dtype), synth.to_f64(d.dY[:ts], L.dtype)
        Bbar, _ = oracle.backward_mask(W, B, P, N, M)
        Wf, Wb = W * B, W[P, :] * Bbar
        g = _best(lambda: X @ Wf.T, reps=2) + _best(lambda: dY[:, P] @ Wb, reps=2)
        add(tall, "gemms_float64", g * T / ts)
        add(t1, "gemms_float64", g * T / ts)        # the library matmul has no one-thread run here: same figure
        if ts < T:
            samples.append(f"{L.name}: float64 GEMMs on {ts} of the {T} tokens, scaled")
        # the oracle's own triple loop on 4096 sampled outputs, per output element (context)
        r = np.random.default_rng(5)
        tt, ii = r.integers(0, ts, 4096), r.integers(0, I, 4096)
        t1["loop_gemm_ns_per_output"] = round(_best(lambda: oracle.gemm_fwd_at(X, W, B, tt, ii), reps=1) * 1e6 / 4096, 1)
        del W, B, X, dY, Wf, Wb, Bbar
    pool.shutdown()
    loop_ns = t1.pop("loop_gemm_ns_per_output")
    return {"value": round(sum(tall.values()), 1), "unit": "ms", "cores": int(cores), "kind": "oracle",
            "single_thread_ms": round(sum(t1.values()), 1),
            "steps_ms_1_thread": {k: round(v, 1) for k, v in t1.items()},
            "steps_ms_all_cores": {k: round(v, 1) for k, v in tall.items()},
            "loop_gemm_ns_per_output": loop_ns,
            "sample": "one step of the same workload; " + ("; ".join(samples) if samples else "every step at full size")
                      + "; the float64 GEMMs are library matmuls on all cores in both columns"}


def all_layers(args):
    """Network aggregate (not the headline line): one pass over every layer of a configuration,
    each stage timed over `steps` back-to-back calls with HIP events; prints one JSON line with
    per-stage totals in microseconds and the per-layer rows."""
    import torch
    from paper_2302_06058_amd import synth
    rows, tot = [], {}
    for layer in synth.get_config(args.config):
        data = synth.gen_layer(layer)
        e = 2 if layer.dtype == "bf16" else 4
        per_copy = e * layer.T * (layer.I + layer.J) * 2
        copies = max(2, min(9, -(-(1 << 29) // per_copy)))
        run = LayerRun(layer, data, copies)
        run.step(0)
        torch.cuda.synchronize()
        row = {"layer": layer.name, "I": layer.I, "J": layer.J, "T": layer.T, "nm": f"{layer.N}:{layer.M}"}
        for name, fn in run.stages:
            for i in range(max(args.warmup, args.steps)):      # as long as the timed run: clocks settle
                fn(i % copies)
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            a.record()
            for i in range(args.steps):
                fn(i % copies)
            b.record()
            torch.cuda.synchronize()
            row[name] = round(a.elapsed_time(b) * 1e3 / args.steps, 2)
            tot[name] = tot.get(name, 0.0) + row[name]
        rows.append(row)
        del run, data
        torch.cuda.empty_cache()
    print(json.dumps({"metric": "Bi-Mask hot path, sum over all layers of the configuration", "unit": "us",
                      "config": args.config, "steps": args.steps, "n_layers": len(rows),
                      "value": round(sum(tot.values()), 1), "stage_totals_us": {k: round(v, 1) for k, v in tot.items()},
                      "layers": rows}), flush=True)


def grouped_network(args):
    """Forward masks, searches and backward masks of every layer of a configuration, issued the way a
    training step can issue them (Alg. 1 treats layers independently): one grouped call per stage for the
    whole network, against the same stages as one call per layer.  Microseconds per pass over the network."""
    import torch
    import paper_2302_06058_amd as bm
    from paper_2302_06058_amd import synth
    from helpers import to_dev, i32_dev
    layers = synth.get_config(args.config)
    by_nm = {}
    for L in layers:
        by_nm.setdefault((L.N, L.M, L.dtype), []).append(L)
    st = torch.cuda.current_stream().cuda_stream
    res = {"forward_mask_compress": [0.0, 0.0], "perm_search": [0.0, 0.0], "backward_mask_compress": [0.0, 0.0]}
    n_launch_groups = 0
    for (N, M, dts), Ls in by_nm.items():
        code = bm.BF16 if dts == "bf16" else bm.F32
        tdt = torch.bfloat16 if dts == "bf16" else torch.float32
        entries, single = [], {k: [] for k in res}
        for L in Ls:
            W, Pd = to_dev(synth.gen_weights(L), L.dtype), i32_dev(synth.gen_perms(L))
            dev = W.device
            i32 = lambda n: torch.empty((n,), dtype=torch.int32, device=dev)
            nws = max(16, bm.workspace_bytes(bm.WS_PERM_SEARCH, L.I, L.J, 0, L.K, code, N, M))
            e = dict(W=W, B_bits=torch.empty((L.I, bm.mask_words(L.J)), dtype=torch.int32, device=dev),
                     Wf_values=torch.empty((bm.operand_elems(L.I, L.J, N, M),), dtype=tdt, device=dev),
                     Wf_index=i32(max(4, bm.operand_index_words(L.I, L.J, N, M))),
                     perms=Pd, scores=i32(L.K), best=i32(1), best_perm=i32(L.I),
                     workspace=torch.empty((nws,), dtype=torch.uint8, device=dev),
                     Bbar_bits=torch.empty((L.I, bm.mask_words(L.J)), dtype=torch.int32, device=dev),
                     Wb_values=torch.empty((bm.operand_elems(L.J, L.I, N, M),), dtype=tdt, device=dev),
                     Wb_index=i32(max(4, bm.operand_index_words(L.J, L.I, N, M))))
            entries.append(e)
            single["forward_mask_compress"].append(bm.prepare("bimask_forward_mask_compress", W, L.I, L.J, L.J, code, N, M,
                                                              e["B_bits"], e["Wf_values"], e["Wf_index"], st))
            single["perm_search"].append(bm.prepare("bimask_perm_search", e["B_bits"], L.I, L.J, N, M, Pd, L.K, e["scores"],
                                                    e["best"], e["best_perm"], e["workspace"], nws, st))
            single["backward_mask_compress"].append(bm.prepare("bimask_backward_mask_compress", W, L.I, L.J, L.J, code, N, M,
                                                               e["B_bits"], e["best_perm"], e["Bbar_bits"], e["Wb_values"],
                                                               e["Wb_index"], st))
        arr = bm.group_layers(entries)
        K = Ls[0].K
        grouped = {"forward_mask_compress": lambda: bm.bimask_forward_mask_compress_group(arr, code, N, M),
                   "perm_search": lambda: bm.bimask_perm_search_group(arr, N, M, K),
                   "backward_mask_compress": lambda: bm.bimask_backward_mask_compress_group(arr, code, N, M)}
        n_launch_groups += 1
        for name in res:
            for which, fn in ((0, lambda: [c() for c in single[name]]), (1, grouped[name])):
                for _ in range(max(args.warmup, args.steps)):
                    fn()
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                torch.cuda.synchronize()
                a.record()
                for _ in range(args.steps):
                    fn()
                b.record()
                torch.cuda.synchronize()
                res[name][which] += a.elapsed_time(b) * 1e3 / args.steps
    print(json.dumps({"metric": "mask and search steps of a whole network, per-layer calls vs grouped calls", "unit": "us",
                      "config": args.config, "n_layers": len(layers), "steps": args.steps,
                      "per_layer_calls_us": {k: round(v[0], 1) for k, v in res.items()},
                      "grouped_calls_us": {k: round(v[1], 1) for k, v in res.items()},
                      "sum_per_layer_us": round(sum(v[0] for v in res.values()), 1),
                      "sum_grouped_us": round(sum(v[1] for v in res.values()), 1)}), flush=True)


def network_step(args):
    """The hot path over a whole network, end to end, the way a training step issues it: forward masks of
    all layers (grouped), forward GEMM per layer, searches (grouped), backward masks (grouped), backward
    GEMM per layer.  All layers' buffers are resident (one copy each: a pass moves far more than the
    last-level cache holds).  Milliseconds per pass, with and without the search."""
    import torch
    import paper_2302_06058_amd as bm
    from paper_2302_06058_amd import synth
    layers = synth.get_config(args.config)
    # everything on one side stream (default priority): the calls are bound to the stream that is current when
    # the buffers are set up, and a HIP graph cannot be captured from the legacy default stream
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        runs = [LayerRun(L, synth.gen_layer(L), 1) for L in layers]
        groups = {}
        for r in runs:
            L = r.layer
            groups.setdefault((L.N, L.M, r.dt, L.K), []).append(r)
        garr = {}
        for key, rs in groups.items():
            garr[key] = bm.group_layers([dict(W=r.W, B_bits=r.B, Wf_values=r.vf, Wf_index=r.xf, perms=r.perms, scores=r.scores,
                                              best=r.best, best_perm=r.P, workspace=r.ws_perm, Bbar_bits=r.Bbar,
                                              Wb_values=r.vb, Wb_index=r.xb) for r in rs])

        def one_pass(search):
            for (N, M, dt, K), arr in garr.items():
                bm.bimask_forward_mask_compress_group(arr, dt, N, M)
            for r in runs:
                r.c_gemm_fwd[0]()
            for (N, M, dt, K), arr in garr.items():
                if search:
                    bm.bimask_perm_search_group(arr, N, M, K)
                bm.bimask_backward_mask_compress_group(arr, dt, N, M)
            for r in runs:
                r.c_gemm_bwd[0]()

        def timed(fn):
            for _ in range(max(2, args.warmup // 4)):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) * 1e3 / args.steps

        one_pass(True)
        ms_with, ms_without = timed(lambda: one_pass(True)), timed(lambda: one_pass(False))
        # the same pass recorded once as a HIP graph and replayed: no per-launch host work between the ~120 kernels.
        # The library allocates nothing and records no memset, so the whole pass captures; outputs of a replay are
        # compared with the eager pass below.
        torch.cuda.synchronize()
        eager = [(r.Y[0].clone(), r.dX[0].clone(), r.P.clone()) for r in runs]
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            one_pass(True)
        ms_graph = timed(graph.replay)
        same = all(torch.equal(r.Y[0], e[0]) and torch.equal(r.dX[0], e[1]) and torch.equal(r.P, e[2])
                   for r, e in zip(runs, eager))
    flops = sum(2 * 2 * L.T * L.I * L.J for L in layers)
    print(json.dumps({"metric": "Bi-Mask step over all layers of the configuration (grouped masks + searches, per-layer GEMMs)",
                      "unit": "ms", "config": args.config, "n_layers": len(layers), "steps": args.steps,
                      "ms_per_pass": round(ms_with, 4), "ms_per_pass_without_search": round(ms_without, 4),
                      "ms_per_pass_search_every_delta_t": round(ms_without + (ms_with - ms_without) / args.delta_t, 4),
                      "ms_per_pass_hip_graph": round(ms_graph, 4), "hip_graph_equals_eager": bool(same),
                      "dense_equiv_tflops": round(flops / (ms_with * 1e-3) / 1e12, 1)}), flush=True)


def gradient_gap(args):
    """What the permutation is for (Sec. 3.3): g-bar(X) of Eq. (10) against g(X) = g(Y) (B .* W) of Eq. (5) on one
    layer, for the identity and for the best of K random permutations, with the share of eligible N:M
    blocks.  Masks, search and g-bar(X) come from the library.  The exact gradient of Eq. (5) is context
    computed here by a plain torch fp32 matmul (it is not a call of the library); the figure is tied to the
    CPU oracle's float64 gap by tests/test_gpu_parity_small.py::test_gradient_gap_against_the_oracle."""
    import torch
    import paper_2302_06058_amd as bm
    from paper_2302_06058_amd import synth
    from helpers import to_dev, i32_dev
    L = synth.get_config(args.config)[max(args.layer, 0)]
    N, M, I, J = L.N, L.M, L.I, L.J
    T = min(L.T, 4096)
    W = to_dev(synth.gen_weights(L), L.dtype)
    dY = to_dev(synth.gen_out_grad(L, T), L.dtype)
    B = bm.bimask_forward_mask(W, N, M)
    shifts = torch.arange(32, device=W.device, dtype=torch.int32)
    unpack = lambda bits: ((bits.unsqueeze(-1) >> shifts) & 1).reshape(bits.shape[0], -1)[:, :J].float()
    exact = dY.float() @ (W.float() * unpack(B))                      # Eq. (5)
    den = float(exact.norm())
    rows = []

    def gap(P):
        Bbar, vb, ib = bm.bimask_backward_mask_compress(W, N, M, B, P)
        approx = bm.bimask_sparse_gemm_bwd(dY, P, vb, ib, I, J, N, M).float()
        kept = float(unpack(Bbar).sum() / unpack(B).sum())
        return float((approx - exact).norm()) / den, kept

    g0, kept0 = gap(None)
    ident = torch.arange(I, dtype=torch.int32, device=W.device).reshape(1, I)
    sc0, _, _ = bm.bimask_perm_search(B, I, J, N, M, ident)
    blocks = (I // M) * J
    rows.append({"permutation": "identity", "eligible_block_share": round(int(sc0[0]) / blocks, 4),
                 "kept_share_of_forward_mask": round(kept0, 4), "relative_gap": round(g0, 4)})
    rng = np.random.default_rng([L.seed, 99])
    for K in (10, 100, 1000):
        perms = i32_dev(np.stack([rng.permutation(I) for _ in range(K)]).astype(np.int32))
        scores, best, P = bm.bimask_perm_search(B, I, J, N, M, perms)
        g, kept = gap(P)
        rows.append({"permutation": f"best of {K}", "eligible_block_share": round(int(scores.max()) / blocks, 4),
                     "kept_share_of_forward_mask": round(kept, 4), "relative_gap": round(g, 4)})
    print(json.dumps({"metric": "||g-bar(X) - g(X)|| / ||g(X)||  (Eq. 10 vs Eq. 5)", "layer": L.name, "I": I, "J": J, "T": T,
                      "nm": f"{N}:{M}", "rows": rows}), flush=True)


def refine_report(args):
    """A permutation better than the best of K random ones (the paper's Limitations name it as future work): hill
    climbing over S random exchange proposals from the search's winner, on one layer.  Reports the time of the
    refinement call, the eligible-block share and the gap of Eq. (10)'s g-bar(X) to Eq. (5)'s g(X)."""
    import torch
    import paper_2302_06058_amd as bm
    from paper_2302_06058_amd import synth
    from helpers import to_dev, i32_dev
    L = synth.get_config(args.config)[max(args.layer, 0)]
    N, M, I, J = L.N, L.M, L.I, L.J
    T = min(L.T, 4096)
    W = to_dev(synth.gen_weights(L), L.dtype)
    dY = to_dev(synth.gen_out_grad(L, T), L.dtype)
    B = bm.bimask_forward_mask(W, N, M)
    shifts = torch.arange(32, device=W.device, dtype=torch.int32)
    unpack = lambda bits: ((bits.unsqueeze(-1) >> shifts) & 1).reshape(bits.shape[0], -1)[:, :J].float()
    exact = dY.float() @ (W.float() * unpack(B))                      # Eq. (5)
    den = float(exact.norm())
    blocks = (I // M) * J

    def gap(P):
        Bbar, vb, ib = bm.bimask_backward_mask_compress(W, N, M, B, P)
        approx = bm.bimask_sparse_gemm_bwd(dY, P, vb, ib, I, J, N, M).float()
        return float((approx - exact).norm()) / den, float(unpack(Bbar).sum() / unpack(B).sum())

    rng = np.random.default_rng([L.seed, 99])
    perms = i32_dev(np.stack([rng.permutation(I) for _ in range(L.K)]).astype(np.int32))
    scores, best, P = bm.bimask_perm_search(B, I, J, N, M, perms)
    start = int(scores.max())
    g, kept = gap(P)
    rows = [{"proposals": 0, "us": 0.0, "kept": 0, "eligible_block_share": round(start / blocks, 4),
             "kept_share_of_forward_mask": round(kept, 4), "relative_gap": round(g, 4)}]
    out = torch.empty_like(P)
    res = torch.empty((2,), dtype=torch.int32, device=W.device)
    for mult in (1, 4, 16, 64):
        S = mult * I
        swaps = i32_dev(rng.integers(0, I, size=(S, 2)).astype(np.int32))
        call = bm.prepare("bimask_perm_refine", B, I, J, N, M, P, swaps, S, out, res,
                          torch.cuda.current_stream().cuda_stream)
        for _ in range(2):
            call()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(args.steps):
            call()
        b.record()
        torch.cuda.synchronize()
        us = a.elapsed_time(b) * 1e3 / args.steps
        g, kept = gap(out)
        r = res.cpu().numpy()
        rows.append({"proposals": S, "us": round(us, 1), "proposals_per_us": round(S / us, 2), "kept": int(r[1]),
                     "eligible_block_share": round((start + int(r[0])) / blocks, 4),
                     "kept_share_of_forward_mask": round(kept, 4), "relative_gap": round(g, 4)})
    print(json.dumps({"metric": "refinement of the best of K = %d random permutations by S random exchange proposals" % L.K,
                      "layer": L.name, "I": I, "J": J, "T": T, "nm": f"{N}:{M}", "steps": args.steps, "rows": rows}),
          flush=True)


def refine_network(args):
    """Refinement of every layer's permutation after the search, S = 4 I random exchange proposals per layer:
    one call per layer (one workgroup busy at a time) against one grouped call (one workgroup per layer, all at once)."""
    import torch
    import paper_2302_06058_amd as bm
    from paper_2302_06058_amd import synth
    from helpers import to_dev, i32_dev
    layers = synth.get_config(args.config)
    by_nm = {}
    for L in layers:
        by_nm.setdefault((L.N, L.M, L.K), []).append(L)
    out = {}
    for (N, M, K), Ls in by_nm.items():
        entries, calls = [], []
        blocks = gain0 = 0
        for L in Ls:
            W = to_dev(synth.gen_weights(L), L.dtype)
            rng = np.random.default_rng([L.seed, 55])
            perms = i32_dev(np.stack([rng.permutation(L.I) for _ in range(K)]).astype(np.int32))
            swaps = i32_dev(rng.integers(0, L.I, size=(4 * L.I, 2)).astype(np.int32))
            e = dict(W=W, B_bits=bm.bimask_forward_mask(W, N, M), perms=perms, swaps=swaps,
                     scores=torch.empty((K,), dtype=torch.int32, device=W.device),
                     best=torch.empty((1,), dtype=torch.int32, device=W.device),
                     best_perm=torch.empty((L.I,), dtype=torch.int32, device=W.device),
                     refine_result=torch.empty((2,), dtype=torch.int32, device=W.device),
                     workspace=torch.empty((max(16, bm.workspace_bytes(bm.WS_PERM_SEARCH, L.I, L.J, 0, K, bm.BF16, N, M)),),
                                           dtype=torch.uint8, device=W.device))
            entries.append(e)
            blocks += (L.I // M) * L.J
        arr = bm.group_layers(entries)
        bm.bimask_perm_search_group(arr, N, M, K)
        torch.cuda.synchronize()
        start = [e["best_perm"].clone() for e in entries]
        base = sum(int(e["scores"].max()) for e in entries)
        st = torch.cuda.current_stream().cuda_stream
        for e, L in zip(entries, Ls):
            calls.append(bm.prepare("bimask_perm_refine", e["B_bits"], L.I, L.J, N, M, e["best_perm"], e["swaps"],
                                    4 * L.I, e["best_perm"], e["refine_result"], st))

        def reset():
            for e, p0 in zip(entries, start):
                e["best_perm"].copy_(p0)

        def timed(fn):
            ts = []
            for _ in range(max(2, args.steps)):
                reset()
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                torch.cuda.synchronize()
                a.record(); fn(); b.record()
                torch.cuda.synchronize()
                ts.append(a.elapsed_time(b))
            return sorted(ts)[len(ts) // 2]

        ms_each = timed(lambda: [c() for c in calls])
        per_layer = [e["best_perm"].clone() for e in entries]
        ms_group = timed(lambda: bm.bimask_perm_refine_group(arr, N, M))
        same = all(torch.equal(e["best_perm"], p) for e, p in zip(entries, per_layer))
        gain = sum(int(e["refine_result"][0]) for e in entries)
        out[f"{N}:{M}"] = {"layers": len(Ls), "proposals": sum(4 * L.I for L in Ls), "ms_one_call_per_layer": round(ms_each, 3),
                           "ms_grouped_call": round(ms_group, 3), "grouped_equals_per_layer": bool(same),
                           "eligible_block_share_before": round(base / blocks, 4),
                           "eligible_block_share_after": round((base + gain) / blocks, 4)}
    print(json.dumps({"metric": "refinement of all layers' permutations (4 I proposals per layer, after the K-candidate search)",
                      "unit": "ms", "config": args.config, "steps": args.steps, "by_pattern": out}), flush=True)


def search_table(args):
    """Whole-network permutation search (forward mask given, K = 100 candidates scored and the best
    picked, per layer) for the five N:M patterns of the paper's Table 6, on the ResNet-50 layer
    shapes.  Rows / columns are padded to multiples of M where a shape needs it (M = 8, 16)."""
    import torch
    import paper_2302_06058_amd as bm
    from paper_2302_06058_amd import synth
    from helpers import to_dev, i32_dev
    out, out_grouped = {}, {}
    for (N, M) in [(2, 4), (4, 8), (1, 4), (2, 8), (1, 16)]:
        total_us, launches = 0.0, 0
        entries = []
        for L in synth.config3(N, M):
            Ip = (L.I + M - 1) // M * M
            Wh = synth.gen_weights(L)
            if Ip != L.I:                                  # fc: 1000 rows -> 1008 for M = 16 (zero rows)
                Wh = np.concatenate([Wh, np.zeros((Ip - L.I, L.J), dtype=Wh.dtype)])
            rng = np.random.default_rng([L.seed, 77])
            perms = np.stack([rng.permutation(Ip) for _ in range(L.K)]).astype(np.int32)
            W, Pd = to_dev(Wh, L.dtype), i32_dev(perms)
            B = bm.bimask_forward_mask(W, N, M)
            scores = torch.empty((L.K,), dtype=torch.int32, device=W.device)
            best = torch.empty((1,), dtype=torch.int32, device=W.device)
            P = torch.empty((Ip,), dtype=torch.int32, device=W.device)
            nws = max(16, bm.workspace_bytes(bm.WS_PERM_SEARCH, Ip, L.J, 0, L.K, bm.BF16, N, M))
            ws = torch.empty((nws,), dtype=torch.uint8, device=W.device)
            call = bm.prepare("bimask_perm_search", B, Ip, L.J, N, M, Pd, L.K, scores, best, P, ws, nws,
                              torch.cuda.current_stream().cuda_stream)
            for _ in range(max(args.warmup, args.steps)):
                call()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            a.record()
            for _ in range(args.steps):
                call()
            b.record()
            torch.cuda.synchronize()
            total_us += a.elapsed_time(b) * 1e3 / args.steps
            launches += 1
            entries.append(dict(W=W, B_bits=B, perms=Pd, scores=scores, best=best, best_perm=P, workspace=ws))
        out[f"{N}:{M}"] = round(total_us / 1e3, 4)
        # the same 54 searches through the grouped entry point
        arr = bm.group_layers(entries)
        for _ in range(max(args.warmup, args.steps)):
            bm.bimask_perm_search_group(arr, N, M, 100)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(args.steps):
            bm.bimask_perm_search_group(arr, N, M, 100)
        b.record()
        torch.cuda.synchronize()
        out_grouped[f"{N}:{M}"] = round(a.elapsed_time(b) / args.steps, 4)
    print(json.dumps({"metric": "permutation search, all 54 ResNet-50 layers, K = 100 (one search per layer)",
                      "unit": "ms", "steps": args.steps, "layers": launches, "search_ms": out, "search_ms_grouped_calls": out_grouped,
                      "paper_table6_seconds_a100": {"2:4": 15.5, "4:8": 14.3, "1:4": 13.6, "2:8": 15.7, "1:16": 15.0},
                      "note": "the paper does not say how many searches its figure covers"}), flush=True)


def only_stage(args):
    """One stage repeated back to back (operands warm in the last-level cache where they fit): the stand-alone
    figure beside the in-sequence one of the step.  Microseconds per call, per matrix."""
    import torch
    from paper_2302_06058_amd import synth
    out = {}
    for L in pick_layers(args.config, args.layer):
        run = LayerRun(L, synth.gen_layer(L), 2)
        run.step(0)
        fn = dict(run.stages)[args.only_stage]
        for i in range(args.warmup):
            fn(i % 2)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for i in range(args.steps):
            fn(i % 2)
        b.record()
        torch.cuda.synchronize()
        alg = algorithmic(L)[args.only_stage]
        us = a.elapsed_time(b) * 1e3 / args.steps
        out[L.name] = {"us": round(us, 2), "algorithmic_GBs": round(alg["bytes"] / us / 1e3, 1),
                       "dense_equiv_TFLOPs": round(alg["flops"] / us / 1e6, 1)}
        del run
        torch.cuda.empty_cache()
    print(json.dumps({"metric": f"stand-alone repeats of stage {args.only_stage}", "config": args.config, "steps": args.steps,
                      "matrices": out}), flush=True)


def pick_layers(config, layer):
    """Layers that make up one step: all layers of configs 1, 2 and 5 (config 5 = the two matrices of the MLP
    block), one layer of configs 3 and 4 (their whole-network steps are --network-step / --all-layers)."""
    from paper_2302_06058_amd import synth
    cfg = synth.get_config(config)
    if layer >= 0:
        return [cfg[layer]]
    return cfg if config in (1, 2, 5) else [cfg[0]]


def measured_traffic(config):
    """HBM bytes per launch of a stage's kernel from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs kept under
    profiles/ (lines `traffic_bytes_per_launch <stage> <bytes>` of bench_config<N>_hbm_traffic.txt, already scaled
    by the copy-kernel calibration stated there); None where no such run is on file."""
    path = os.path.join(ROOT, "profiles", f"bench_config{config}_hbm_traffic.txt")
    out = {}
    if os.path.exists(path):
        with open(path) as f:
            for line in f:
                w = line.split()
                if len(w) == 3 and w[0] == "traffic_bytes_per_launch":
                    out[w[1]] = int(w[2])
    return out


def dense_context(runs, copies, reps=10):
    """Context only, never part of `value`: the DENSE bf16 GEMMs of the same shapes through the library behind
    torch.matmul, on the same rotating activations -- the forward and backward products the sparse GEMMs replace
    (Eq. 3, Eq. 10 without masks) and the weight gradient dW = dY^T X, which the method leaves dense (Sec. 3.1,
    Limitations).  Microseconds per call, HIP events around each call."""
    import torch
    out = {}
    for r in runs:
        if r.W.dtype != torch.bfloat16:
            continue
        Wt = r.W.t()
        ops = {"dense_fwd  X W^T": lambda c: torch.matmul(r.X[c], Wt),
               "dense_bwd  dY W": lambda c: torch.matmul(r.dY[c], r.W),
               "dense_dW  dY^T X": lambda c: torch.matmul(r.dY[c].t(), r.X[c])}
        d = {}
        for name, fn in ops.items():
            for i in range(3):
                fn(i % copies)
            pairs = []
            for i in range(reps):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record(); fn(i % copies); b.record()
                pairs.append((a, b))
            torch.cuda.synchronize()
            ts = sorted(a.elapsed_time(b) * 1e3 for a, b in pairs)
            d[name] = round(ts[len(ts) // 2], 2)
        out[r.layer.name] = d
    torch.cuda.empty_cache()
    return out


def measure(args, config, layer_sel, steps, warmup, with_cpu, with_context=False):
    """Times `steps` steps of the chosen workload and returns the fields of the JSON line."""
    import torch
    import paper_2302_06058_amd as bm
    from paper_2302_06058_amd import synth
    layers = pick_layers(config, layer_sel)
    datas = [synth.gen_layer(L) for L in layers]
    e = 2 if layers[0].dtype == "bf16" else 4
    per_copy = sum(e * L.T * (L.I + L.J) * 2 for L in layers)
    # enough rotating copies that a step never finds its activations in the 256 MB last-level cache
    copies = args.copies or max(2, min(16, -(-(1 << 30) // per_copy)))
    runs = [LayerRun(L, d, copies) for L, d in zip(layers, datas)]
    algs = [algorithmic(L) for L in layers]
    stage_names = [n for n, _ in runs[0].stages]

    def step(i):
        for r in runs:
            r.step(i)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()

    # -- per-stage breakdown (HIP events on the launch stream), outside the timed region
    ev = lambda: torch.cuda.Event(enable_timing=True)
    stage_us = []
    for r in runs:
        d = {}
        for name, fn in r.stages:
            pairs = []
            for i in range(args.breakdown_reps):
                a, b = ev(), ev()
                a.record(); fn(i % copies); b.record()
                pairs.append((a, b))
            torch.cuda.synchronize()
            ts = sorted(a.elapsed_time(b) * 1e3 for a, b in pairs)
            d[name] = {"avg": sum(ts) / len(ts), "min": ts[0], "median": ts[len(ts) // 2]}
        stage_us.append(d)

    # -- dominant kernel.  Among the two stages with the largest roofline time (summed over the layers of the
    #    step) the slower one; a backward stage that runs TWO kernels (the separate g(Y) column gather, then the
    #    same GEMM kernel as the forward stage with the same flop count) is not one kernel's duration, so the
    #    kernel is then timed where it runs alone: on the forward stage.
    tot_alg = {n: {"bytes": sum(a[n]["bytes"] for a in algs), "flops": sum(a[n]["flops"] for a in algs)} for n in stage_names}
    roof_t = {k: max(v["bytes"] / (HBM_PEAK_GBS * 1e9), v["flops"] / (MFMA_BF16_PEAK_TFLOPS * 1e12)) for k, v in tot_alg.items()}
    top2 = sorted(roof_t, key=roof_t.get, reverse=True)[:2]
    dominant = max(top2, key=lambda k: sum(d[k]["median"] for d in stage_us))
    two_kernels = any(bm.workspace_bytes(bm.WS_GEMM_BWD, L.I, L.J, L.T, 0, r.dt, L.N, L.M) > 0 for L, r in zip(layers, runs))
    if dominant == "sparse_gemm_bwd" and two_kernels:
        dominant = "sparse_gemm_fwd"

    # -- timed region: exactly `steps` steps, events only around the dominant stage, in one step out of EVENT_EVERY
    dom_pairs = []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        rr = i % copies
        for r in runs:
            for name, fn in r.stages:
                if name == dominant and i % EVENT_EVERY == 0:
                    a, b = ev(), ev()
                    a.record(); fn(rr); b.record()
                    dom_pairs.append((a, b))
                else:
                    fn(rr)
    issue_ms = (time.perf_counter() - t0) * 1e3 / steps       # host time to enqueue one step
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
    dom_us = sum(a.elapsed_time(b) for a, b in dom_pairs) * 1e3 / len(dom_pairs)     # average per launch
    # what an event pair reads with nothing between its two records, in the same queue state (right after a
    # kernel): the part of dom_us that is marker processing, not kernel time.  Reported, never subtracted.
    empty_pairs = []
    for i in range(20):
        runs[0].stages[0][1](i % copies)
        a, b = ev(), ev()
        a.record(); b.record()
        empty_pairs.append((a, b))
    torch.cuda.synchronize()
    empty_us = sorted(a.elapsed_time(b) * 1e3 for a, b in empty_pairs)[len(empty_pairs) // 2]

    # -- secondary figure: the step as Alg. 1 runs it between two searches (P kept for delta-T steps)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for i in range(steps):
        rr = i % copies
        for r in runs:
            for name, fn in r.stages:
                if name != "perm_search":
                    fn(rr)
    torch.cuda.synchronize()
    ms_no_search = (time.perf_counter() - t1) * 1e3 / steps

    # per launch: the layers of a step launch the dominant kernel once each; bytes / flops averaged like the time
    dom_bytes = tot_alg[dominant]["bytes"] / len(layers)
    dom_flops = tot_alg[dominant]["flops"] / len(layers)
    gbs = dom_bytes / (dom_us * 1e-6) / 1e9
    tfl = dom_flops / (dom_us * 1e-6) / 1e12
    t_hbm, t_mfma = dom_bytes / (HBM_PEAK_GBS * 1e9), dom_flops / (MFMA_BF16_PEAK_TFLOPS * 1e12)
    if t_hbm >= t_mfma:
        roof = {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(gbs / HBM_PEAK_GBS, 4)}
    else:
        # dense-equivalent flops 2 T I J (the convention of the stated target); the sparse cores execute half of them
        roof = {"bound": "mfma", "achieved": round(tfl, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(tfl / MFMA_BF16_PEAK_TFLOPS, 4), "flops": "dense-equivalent 2*T*I*J",
                "frac_executed_flops": round(tfl / 2 / MFMA_BF16_PEAK_TFLOPS, 4) if layers[0].N <= 2 else None}
    roof.update({"traffic": measured_traffic(config).get(dominant), "kernel": dominant,
                 "launches_per_step": len(layers), "avg_us": round(dom_us, 2),
                 "empty_event_pair_us": round(empty_us, 2),
                 "algorithmic_bytes": int(dom_bytes), "dense_equiv_tflops": round(tfl, 1)})

    def wl(L):
        return f"{L.name} W {L.I}x{L.J}, T={L.T}, {L.N}:{L.M}, K={L.K}, {L.dtype}"
    out = {
        "ms_per_step": round(ms_per_step, 5),
        "config": {"workload": f"config{config}: " + " + ".join(wl(L) for L in layers)
                               + ("  (one step = the whole path over every matrix listed)" if len(layers) > 1 else ""),
                   "rotating_copies": copies},
        "roofline": roof,
        "stages_us": {L.name: {k: {kk: round(vv, 2) for kk, vv in v.items()} for k, v in d.items()}
                      for L, d in zip(layers, stage_us)},
        "stages_sum_us": round(sum(v["avg"] for d in stage_us for v in d.values()), 2),
        "host_enqueue_ms_per_step": round(issue_ms, 5),
        "amortised": {"delta_t": args.delta_t, "ms_per_step_without_search": round(ms_no_search, 5),
                      "ms_per_step_search_every_delta_t": round(ms_no_search + max(ms_per_step - ms_no_search, 0.0) / args.delta_t, 5)},
    }
    if with_context:
        out["context"] = {"dense_library_gemm_us": dense_context(runs, copies),
                          "note": "torch.matmul on dense bf16 operands of the same shapes, median of 10 calls; outside the timed "
                                  "region and not part of value: what the sparse forward / backward GEMMs replace, and the dense "
                                  "weight gradient the method keeps"}
    del runs
    torch.cuda.empty_cache()
    if with_cpu:
        out["cpu_baseline"] = cpu_baseline(layers, datas)
    return out, layers


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures the single-GPU hot path only: this build has no multi-GPU path "
              "(run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2302_06058_amd as bm
    bm.lib()                                   # fail loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    if args.only_stage:
        if args.config is None:
            args.config = 5
        return only_stage(args)
    headline = not (args.all_layers or args.search_table or args.grouped or args.gradient_gap or args.refine
                    or args.refine_network or args.network_step)
    if args.config is None:
        args.config = 5 if headline else 2
    if args.all_layers:
        return all_layers(args)
    if args.search_table:
        return search_table(args)
    if args.grouped:
        return grouped_network(args)
    if args.gradient_gap:
        return gradient_gap(args)
    if args.refine:
        return refine_report(args)
    if args.refine_network:
        return refine_network(args)
    if args.network_step:
        return network_step(args)

    res, layers = measure(args, args.config, args.layer, args.steps, args.warmup, not args.no_cpu_baseline,
                          with_context=not args.no_context)
    out = {
        "metric": "Bi-Mask per-layer step time (mask+perm+fwd/bwd GEMM)",
        "value": res["ms_per_step"], "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"], "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": layers[0].dtype, "data": "synthetic",
    }
    out.update({k: v for k, v in res.items() if k != "ms_per_step"})
    if args.config == 5 and not args.no_secondary:
        # the HBM-bound ResNet-50 layer3 3x3 convolution (config 2) beside the headline, same protocol
        sec, _ = measure(args, 2, -1, max(args.steps, 200), max(args.warmup, 20), False)
        out["secondary"] = {"config2": sec}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
