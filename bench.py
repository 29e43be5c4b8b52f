#!/usr/bin/env python3
"""Benchmark of the Dictionary Annealing sweep (arXiv 1509.05194, Sec. 3.1) on one MI355X.

One step = one pass of the whole hot path over the SIFT-shaped workload: a full DA sweep
(heat, T Lloyd iterations of assign + centroid update, re-encode, new residue, for each of
the M dictionaries) over N resident vectors, plus greedy encoding of 10,000 held-out queries.
Prints ONE JSON line.  Inputs are seeded synthetic stand-ins shaped like 128-d SIFT
descriptors (integer-valued in [0,255], ~30 % zeros), already in HBM when timing starts.

How much work a sweep with the exact shortcuts does depends on how settled the dictionaries are, so every
timed step restores a named state first (outside the timer) and all steps of one figure time the SAME sweep:
  fresh_sweep         from all-zero dictionaries (seeded with rows of the residue);
  first_anneal_sweep  the sweep that follows it -- the headline `value`;
  converged_sweep     the sweep after CONVERGED_AFTER sweeps.
`unpruned` times first_anneal_sweep with every assignment and every centroid sum over all vectors
(state-independent work, identical results).  Further keys carry short runs of the other configurations.
"""
import argparse
import json
import sys
import time

import numpy as np

PEAK_FP32_MFMA_TFLOPS = 157.3     # MI355X dense fp32 matrix peak
PEAK_BF16_MFMA_TFLOPS = 2500.0    # MI355X dense bf16 matrix peak
PEAK_HBM_GBS = 8000.0             # MI355X HBM3E peak
CONVERGED_AFTER = 8                # sweeps before the one `converged_sweep` times
MANY_SWEEPS = 20                   # annealing sweeps of the hclae_anneal figure

# HBM bytes per N=1M launch of the assign kernel from two rocprofv3 --pmc runs (FETCH_SIZE 250,672.6 KiB
# x 2.000, WRITE_SIZE 16,135.5 KiB x 1.000; factors from a 512 MB device copy in the same runs), recorded
# in profiles/da_sweep_sift1m_counters.md: the launches that also store the distance bounds.  Algorithmic
# bytes are 521e6 (x', codes, bounds).
ASSIGN_TRAFFIC_BYTES = 5.299e8   # (250672.6 * 2.000 + 16135.5) KiB
# the same for the D-chunked kernel at N=1M, D=960 (profiles/da_sweep_gist1m_counters.md); algorithmic 3.841e9
ASSIGN_TRAFFIC_BYTES_GIST = 4.035e9   # (1962277.4 * 2.000 + 16313.4) KiB


class State:
    """Dictionaries, codes and residues of one learner on the device, with named snapshots."""

    def __init__(self, torch, Xg, M, K):
        N, D = Xg.shape
        self.torch = torch
        self.C = torch.zeros((M, K, D), dtype=torch.float32, device=Xg.device)
        self.codes = torch.zeros((N, M), dtype=torch.uint8, device=Xg.device)
        self.r = Xg.clone()                 # all-zero dictionaries: residue = x
        self.snaps = {}

    def save(self, name):
        self.snaps[name] = (self.C.clone(), self.codes.clone(), self.r.clone())

    def restore(self, name):
        C, codes, r = self.snaps[name]
        self.C.copy_(C)
        self.codes.copy_(codes)
        self.r.copy_(r)

    def drop(self, name):
        self.snaps.pop(name, None)


def timed_steps(torch, state, name, run, steps, warmup):
    """Mean seconds of `run()` over `steps` steps, each from the restored state `name` (restore untimed)."""
    for _ in range(warmup):
        state.restore(name)
        run()
    total = 0.0
    for _ in range(steps):
        state.restore(name)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run()
        torch.cuda.synchronize()
        total += time.perf_counter() - t0
    return total / steps


def sweep_bench(args, torch, hclae, synth, dev, gist, extras):
    N, D, M, K, T, Q = args.n, (960 if gist else 128), args.m, 256, args.iters, args.queries
    t_gen = time.perf_counter()
    gen = synth.gist_like if gist else synth.sift_like
    X = gen(N, D=D)
    Xq = gen(Q, D=D, seed=synth.SEED_HELDOUT)
    idx = synth.init_indices(N, M, K)
    t_gen = time.perf_counter() - t_gen

    Xg = torch.from_numpy(X).to(dev)
    Xqg = torch.from_numpy(Xq).to(dev)
    st = State(torch, Xg, M, K)
    qcodes = torch.zeros((Q, M), dtype=torch.uint8, device=dev)
    qres = torch.empty((Q, D), dtype=torch.float32, device=dev)
    ctx = hclae.Context(N, D, M, K)
    split = args.contraction == "split"
    ctx.set_contraction(1 if split else 0)
    ctx.set_pruning(not args.no_pruning)
    steps, warmup = args.steps, max(args.warmup, 1)
    side_steps = max(1, min(steps, 5))                       # steps of the figures reported beside the headline

    def step_from_scratch():
        ctx.sweep(st.C, st.codes, st.r, T, init_idx=idx, want_err=False)
        ctx.encode(Xqg, st.C, qcodes, qres)

    def step():
        ctx.sweep(st.C, st.codes, st.r, T, want_err=False)
        ctx.encode(Xqg, st.C, qcodes, qres)

    def step_assign_timed():
        ctx.timing_enable(["assign"])
        ctx.sweep(st.C, st.codes, st.r, T, want_err=False)
        ctx.timing_enable([])
        ctx.encode(Xqg, st.C, qcodes, qres)

    # ---- the named states (nothing here is timed)
    st.save("zero")
    step_from_scratch()
    st.save("after_fresh")
    for _ in range(CONVERGED_AFTER - 1):
        step()
    st.save("converged")
    torch.cuda.synchronize()
    ctx.timing_read()

    # ---- headline: the first annealing sweep
    t_first = timed_steps(torch, st, "after_fresh", step_assign_timed, steps, warmup)
    times = ctx.timing_read()
    E_first = ctx.quant_error(st.r)
    a_ms, a_n = times["assign"]
    # launches of the warm-up steps are in the sums too: same kernel on the same state
    assign_ms = a_ms / max(a_n, 1)
    flops = 2.0 * N * K * D                               # algorithmic flops of one assign launch over all N
    # the split contraction issues three bf16 MFMAs per product: its roofline counts those against the bf16 peak
    mfma_flops = 3.0 * flops if split else flops
    peak = PEAK_BF16_MFMA_TFLOPS if split else PEAK_FP32_MFMA_TFLOPS
    achieved = mfma_flops / (assign_ms * 1e-3) / 1e12

    out = {
        "metric": "DA sweep vectors/sec per stage (D=%d,K=256)" % D,
        "value": N * M / t_first,
        "unit": "vectors/s per stage",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": t_first * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if split else "f32",
        "data": "synthetic",
        "config": {"workload": "%s-shaped: N=%d, D=%d, M=%d, K=256, T=%d Lloyd iterations per stage; one step = the "
                               "first annealing DA sweep after a sweep from all-zero dictionaries (every step "
                               "restarts from that same state, restored outside the timer) + greedy encode of %d "
                               "held-out queries" % ("GIST" if gist else "SIFT", N, D, M, T, Q),
                   "N": N, "D": D, "M": M, "K": K, "iters": T, "queries": Q,
                   "timed_sweep": "first_anneal_sweep",
                   "quant_error_after": E_first},
        "roofline": {"bound": "mfma", "kernel": ("%s (fp32 MFMA distance contraction + argmin; the launches over "
                                                 "all N vectors: with the exact shortcuts on, the first assignment "
                                                 "of each stage, which also stores the distance bounds)"
                                                 % ("k_assign_chunked<8>" if gist else "k_assign_resident<8>")
                                                 if not split else
                                                 "%s (split-bf16 MFMA distance contraction + argmin: three bf16 "
                                                 "MFMAs per product, 6NKD flop per launch against the bf16 peak)"
                                                 % ("k_assign_split_chunked<8>" if gist else "k_assign_split<8>")),
                     "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
                     "frac": achieved / peak,
                     "traffic": (ASSIGN_TRAFFIC_BYTES if (N, D, K) == (1_000_000, 128, 256) else
                                 ASSIGN_TRAFFIC_BYTES_GIST if (N, D, K) == (1_000_000, 960, 256) else None)
                                if not split and not args.no_pruning else None,
                     "avg_launch_ms": assign_ms, "launches": a_n, "flops_per_launch": mfma_flops},
    }

    if not args.no_breakdown:
        # ---- the other named sweeps
        sweeps = {"first_anneal_sweep": {"ms_per_step": t_first * 1e3, "value": N * M / t_first, "steps": steps,
                                         "quant_error_after": E_first}}
        t = timed_steps(torch, st, "zero", step_from_scratch, side_steps, 1)
        sweeps["fresh_sweep"] = {"ms_per_step": t * 1e3, "value": N * M / t, "steps": side_steps,
                                 "quant_error_after": ctx.quant_error(st.r),
                                 "note": "from all-zero dictionaries; the copy of the seed rows from the host and one "
                                         "stream synchronisation are inside the call"}
        t = timed_steps(torch, st, "converged", step, side_steps, 1)
        sweeps["converged_sweep"] = {"ms_per_step": t * 1e3, "value": N * M / t, "steps": side_steps,
                                     "quant_error_after": ctx.quant_error(st.r),
                                     "note": "the sweep after %d sweeps" % CONVERGED_AFTER}
        for v in sweeps.values():
            v["unit"] = "vectors/s per stage"
        if not gist and not args.no_pruning:
            # ---- a run of many annealing sweeps: one hclae_anneal call (every stage starts from the distance bounds
            # its last visit kept) against the same sweeps as separate hclae_sweep calls; the same final state
            def many(n):
                st.restore("after_fresh")
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                ctx.anneal(st.C, st.codes, st.r, T, n, want_err=False)
                torch.cuda.synchronize()
                return time.perf_counter() - t0
            t_all, t_head = many(MANY_SWEEPS), many(MANY_SWEEPS - 4)
            t_all = min(t_all, many(MANY_SWEEPS))
            e_many = ctx.quant_error(st.r)
            st.restore("after_fresh")
            torch.cuda.synchronize()
            each = []
            for _ in range(MANY_SWEEPS):
                t0 = time.perf_counter()
                ctx.sweep(st.C, st.codes, st.r, T, want_err=False)
                torch.cuda.synchronize()
                each.append(time.perf_counter() - t0)
            assert ctx.quant_error(st.r) == e_many, "hclae_anneal ended at another quantization error"
            sweeps["anneal_call"] = {
                "sweeps": MANY_SWEEPS, "ms_total": t_all * 1e3, "ms_total_as_sweep_calls": sum(each) * 1e3,
                "ms_per_sweep_last_4": (t_all - t_head) * 1e3 / 4, "ms_per_sweep_last_4_as_sweep_calls": sum(each[-4:]) * 1e3 / 4,
                "value": N * M * MANY_SWEEPS / t_all, "unit": "vectors/s per stage", "quant_error_after": e_many,
                "note": "annealing sweeps 1..%d after the sweep from all-zero dictionaries, in one hclae_anneal call; "
                        "bit-identical to the separate calls" % MANY_SWEEPS}
        out["sweeps"] = sweeps

        # ---- where the time of the headline step goes: every kernel class bracketed by events, one more step
        st.restore("after_fresh")
        ctx.work_counters(reset=True)
        ctx.timing_enable(hclae.KERNEL_CLASSES)
        ctx.sweep(st.C, st.codes, st.r, T, want_err=False)
        bs = ctx.timing_read()                                  # the sweep alone
        n_assign, n_vec, n_refined = ctx.work_counters(reset=True)
        ctx.encode(Xqg, st.C, qcodes, qres)
        ctx.timing_enable([])
        be = ctx.timing_read()                                  # the encode of the held-out queries
        bt = {c: (bs[c][0] + be[c][0], bs[c][1] + be[c][1]) for c in bs}
        tot = sum(ms for ms, n in bt.values())
        share = {"note": "share of the summed kernel time of one first_anneal_sweep step (events around every launch; "
                         "they lengthen the step itself)", "kernel_ms_total": tot,
                 "classes": {c: {"share": ms / tot, "ms": ms, "launches": n} for c, (ms, n) in bt.items() if n}}
        # what the exact shortcuts leave to the matrix cores, counted on the device (hclae_work_counters)
        act_ms = bs["assign_active"][0]
        act_vec = n_vec - M * N                               # beyond the first assignment of each stage
        share["assignments"] = n_assign
        share["vectors_recomputed"] = n_vec
        share["vectors_recomputed_vs_unpruned"] = n_vec / float((T + 1) * M * N)
        share["vectors_rechecked_fp64"] = n_refined
        scale = (3.0 if split else 1.0) * 2.0 * K * D
        if act_ms > 0 and act_vec > 0:
            tf = scale * act_vec / (act_ms * 1e-3) / 1e12
            share["assign_active_TFLOPs"] = tf
            share["assign_active_frac_mfma"] = tf / peak
        out["time_share"] = share
        # the assign kernel in ALL its launches of the sweep (first assignments over all vectors and pruned ones over
        # the listed vectors): algorithmic flop of the vectors actually recomputed over the time of those launches
        fam_ms = bs["assign"][0] + bs["assign_active"][0]
        if fam_ms > 0:
            tf = scale * n_vec / (fam_ms * 1e-3) / 1e12
            out["roofline"]["all_assign_launches_of_the_sweep"] = {
                "achieved": tf, "frac": tf / peak, "launches": bs["assign"][1] + bs["assign_active"][1],
                "share_of_kernel_time": fam_ms / tot,
                "note": "first assignments of the stages (the entry above) together with the pruned assignments"}

        # ---- every kernel class on its own terms: one converged-state sweep (fused stage boundaries), then the
        # same stages one by one so that heat and cool run as separate passes, then the error reduction
        ctx.timing_enable(hclae.KERNEL_CLASSES)
        ctx.sweep(st.C, st.codes, st.r, T, want_err=False)
        for m in range(M):
            ctx.anneal_stage(m, st.C, st.codes, st.r, T, want_stats=False)
        ctx.quant_error(st.r)
        ctx.timing_enable([])
        bt = ctx.timing_read()
        alg_bytes = {"heat": N * (8 * D + 1 + 1), "cool": N * (8 * D + 1 + 1), "accumulate": N * (4 * D + 1),
                     "error": N * 4 * D, "transition": N * (8 * D + 2 + 2)}
        kernels = {}
        for cls, (ms, n) in bt.items():
            if n == 0:
                continue
            e = {"avg_ms": ms / n, "launches": n}
            if cls in alg_bytes:
                gbs = alg_bytes[cls] / (ms / n * 1e-3) / 1e9
                e.update(achieved_GBs=gbs, frac_hbm=gbs / PEAK_HBM_GBS)
            if cls == "assign":
                tf = mfma_flops / (ms / n * 1e-3) / 1e12
                e.update(achieved_TFLOPs=tf, frac_mfma=tf / peak)
            kernels[cls] = e
        out["kernels"] = kernels

        def variant(setup, undo):
            setup()
            ctx.timing_read()
            ts = timed_steps(torch, st, "after_fresh", step_assign_timed, side_steps, 1)
            v_ms, v_n = ctx.timing_read()["assign"]
            e_v = ctx.quant_error(st.r)
            undo()
            assert e_v == E_first, "variant ended at another quantization error: %r vs %r" % (e_v, E_first)
            return ts, v_ms / max(v_n, 1)

        if not args.no_pruning:
            # the same step without the exact shortcuts: every assignment and centroid sum over all N vectors
            ts, a_ms1 = variant(lambda: ctx.set_pruning(False), lambda: ctx.set_pruning(True))
            tf = flops / (a_ms1 * 1e-3) / 1e12
            out["unpruned"] = {
                "value": N * M / ts, "unit": "vectors/s per stage", "ms_per_step": ts * 1e3, "steps": side_steps,
                "assign_avg_launch_ms": a_ms1,
                ("assign_frac_fp32_mfma_peak" if not split else "assign_algorithmic_TFLOPs"):
                    (tf / PEAK_FP32_MFMA_TFLOPS if not split else tf),
                "note": "hclae_set_pruning(0): all (T+1) assignments and all T centroid sums of a stage over all N "
                        "vectors -- work that does not depend on the state; the same sweep from the same state, "
                        "same dictionaries, codes and residues"}
        if not split:
            # the same step with the optional split-bf16 contraction (hclae_set_contraction 1): identical results
            # by construction (same fp64 decisions), another matrix-core arithmetic
            ts, s_avg = variant(lambda: ctx.set_contraction(1), lambda: ctx.set_contraction(0))
            out["split_bf16_contraction"] = {
                "value": N * M / ts, "unit": "vectors/s per stage", "ms_per_step": ts * 1e3, "steps": side_steps,
                "assign_avg_launch_ms": s_avg,
                "assign_algorithmic_TFLOPs": flops / (s_avg * 1e-3) / 1e12,
                "assign_frac_bf16_mfma_peak": 3.0 * flops / (s_avg * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS,
                "note": "fp32 operands split into two bf16 terms, three bf16 MFMAs per product, fp32 accumulation; the "
                        "same sweep from the same state, same codes, dictionaries and residues as the fp32 kernel"}

    if extras and not gist:
        out["improved_kmeans_stage"] = pca_stage_bench(torch, hclae, synth, ctx, st, idx, N, D, M, K)
    for name in list(st.snaps):
        st.drop(name)

    if not args.no_cpu_baseline:
        import oracle
        # the oracle's stages 0 and 1 of the sweep from all-zero dictionaries, and the GPU's own two stages of
        # the same work (same seeds, exact shortcuts off and on) beside it
        Ns = N if not gist else N // 8                      # about 10-20 s on 16 threads
        Xs = np.ascontiguousarray(X[:Ns])
        Co = np.zeros((M, K, D), np.float64)
        co = np.zeros((Ns, M), np.uint8)
        ro = Xs.astype(np.float64)
        idx_s = synth.init_indices(Ns, M, K)
        tc = time.perf_counter()
        oracle.anneal_stage(0, Co, co, ro, T, idx_s[0])
        oracle.anneal_stage(1, Co, co, ro, T, idx_s[1])
        tc = time.perf_counter() - tc
        out["cpu_baseline"] = {"value": 2 * Ns / tc, "unit": "vectors/s per stage", "cores": oracle.threads(),
                               "kind": "oracle",
                               "sample": "two DA stages (m=0,1 of the sweep from all-zero dictionaries, T=%d, K=256) "
                                         "of the fp64 oracle on %s %d vectors of the same workload, %.1f s"
                                         % (T, "all" if Ns == N else "the first", Ns, tc)}
        del ro, co
        xs_g = torch.from_numpy(Xs).to(dev) if Ns != N else Xg
        same = {}
        for pruned in (True, False):
            ctx.set_pruning(pruned)
            tt = []
            for _ in range(3):
                Cs = torch.zeros((M, K, D), dtype=torch.float32, device=dev)
                cs = torch.zeros((Ns, M), dtype=torch.uint8, device=dev)
                rs = xs_g.clone()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                ctx.anneal_stage(0, Cs, cs, rs, T, init_idx=idx_s[0], want_stats=False)
                ctx.anneal_stage(1, Cs, cs, rs, T, init_idx=idx_s[1], want_stats=False)
                torch.cuda.synchronize()
                tt.append(time.perf_counter() - t0)
            same["pruned" if pruned else "unpruned"] = 2 * Ns / min(tt)
        ctx.set_pruning(not args.no_pruning)
        out["cpu_baseline"]["gpu_same_work_vectors_per_s_per_stage"] = same
    out["host_gen_s"] = t_gen
    ctx.close()
    return out


def pca_stage_bench(torch, hclae, synth, ctx, st, idx, N, D, M, K):
    """Improved k-means of Sec. 3.2 as the cool-down of stage 0 of the sweep from all-zero dictionaries (principal
    axes found inside the library, ten dimension prefixes, one Lloyd iteration each), beside the plain stage with
    the same number of Lloyd iterations."""
    dims = []
    for i in range(1, 11):
        d = int(np.ceil(D ** (i / 10.0) - 1e-9))
        if not dims or d > dims[-1]:
            dims.append(d)
    dims[-1] = D
    xr = torch.empty_like(st.r)
    res = {}
    for kind in ("improved", "plain"):
        tt = []
        for _ in range(3):
            st.restore("zero")
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            if kind == "improved":
                s = ctx.anneal_stage_pca(0, st.C, st.codes, st.r, None, dims, 1, xr, init_idx=idx[0])
            else:
                s = ctx.anneal_stage(0, st.C, st.codes, st.r, len(dims), init_idx=idx[0])
            torch.cuda.synchronize()
            tt.append(time.perf_counter() - t0)
        res[kind] = {"ms_per_stage": min(tt) * 1e3, "vectors_per_s": N / min(tt), "quant_error_after": s["err_after"]}
    # the whole sweep from all-zero dictionaries with either cool-down (hclae_set_cooldown): time and E after each stage
    T = len(dims)
    for kind in ("improved", "plain"):
        ctx.set_cooldown(kind == "improved", 10)
        tt = []
        for _ in range(2):
            st.restore("zero")
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            E = ctx.sweep(st.C, st.codes, st.r, T, init_idx=idx)
            torch.cuda.synchronize()
            tt.append(time.perf_counter() - t0)
        res[kind]["sweep_ms"] = min(tt) * 1e3
        res[kind]["sweep_quant_error_per_stage"] = [float(e) for e in E]
    ctx.set_cooldown(False)
    res["note"] = ("stage 0 from all-zero dictionaries, %d Lloyd iterations either way; improved = covariance on the "
                   "device, eigen-decomposition on the host (inside the call), rotation, prefixes %s, rotation back; "
                   "sweep_*: the whole sweep from all-zero dictionaries (M stages) cooled either way, per-stage "
                   "errors read back inside the timed call" % (len(dims), dims))
    return res


def beam_bench(args, torch, hclae, synth, dev, steps=None):
    """Multi-path encoding of the N resident vectors with L paths under dictionaries learned from scratch by one
    sweep.  Reported beside, not instead of, the sweep benchmark."""
    N, D, M, K, T, L = args.n, 128, args.m, 256, args.iters, args.beam
    steps = steps or args.steps
    X = synth.sift_like(N, D=D)
    Xg = torch.from_numpy(X).to(dev)
    C = torch.zeros((M, K, D), dtype=torch.float32, device=dev)
    codes = torch.zeros((N, M), dtype=torch.uint8, device=dev)
    r = Xg.clone()
    ctx = hclae.Context(N, D, M, K)
    ctx.set_contraction(1 if args.contraction == "split" else 0)
    ctx.sweep(C, codes, r, T, init_idx=synth.init_indices(N, M, K), want_err=False)
    ctx.encode(Xg, C, codes, r)
    e_greedy = ctx.quant_error(r)
    ctx.encode_beam(Xg, C, L, codes, r)
    torch.cuda.synchronize()
    ctx.timing_enable(["beam_score", "beam_expand", "norms"])
    t0 = time.perf_counter()
    for _ in range(steps):
        ctx.encode_beam(Xg, C, L, codes, r)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ctx.timing_enable([])
    times = ctx.timing_read()
    e_beam = ctx.quant_error(r)
    per = (t1 - t0) / steps
    rows = N * (1 + (M - 1) * min(L, K))                  # beam rows scored per encode: 1 path, then L
    flops = 2.0 * rows * K * D
    s_ms, s_n = times["beam_score"]
    x_ms, x_n = times["beam_expand"]
    achieved = flops * steps / (s_ms * 1e-3) / 1e12 if s_ms else None
    ctx.close()
    return {
        "metric": "multi-path encoding vectors/sec (D=128, K=256, M=%d, L=%d)" % (M, L),
        "value": N / per, "unit": "vectors/s", "n_gpus": 1, "steps": steps, "warmup": 1,
        "ms_per_step": per * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "SIFT-shaped: N=%d, D=128, M=%d, K=256; dictionaries from one fresh DA sweep (T=%d); "
                               "one step = multi-path encoding of all N vectors with L=%d" % (N, M, T, L),
                   "quant_error_greedy": e_greedy, "quant_error_multipath": e_beam},
        "roofline": {"bound": "mfma", "kernel": ("k_beam_score_resident<8> (fp32 MFMA scoring of N*L beam rows)"
                                                 if args.contraction == "f32" else
                                                 "k_beam_score_split<8> (split-bf16 MFMA scoring; algorithmic flop "
                                                 "against the fp32 peak for comparison)"),
                     "achieved": achieved, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_FP32_MFMA_TFLOPS if achieved else None, "traffic": None,
                     "flops_per_step": flops},
        "kernels": {"beam_score": {"ms_per_step": s_ms / steps, "launches": s_n},
                    "beam_expand": {"ms_per_step": x_ms / steps, "launches": x_n}},
    }


def online_bench(args, torch, hclae, synth, dev, nchunks=None):
    """Online sweep over uint8 chunks held in pinned host memory: hipMemcpyAsync of chunk i+1 on a side
    stream into one of two staging buffers while chunk i is processed.  A ring of 4 distinct seeded
    chunks stands in for the stream (generating 100 distinct chunks would take minutes of host time)."""
    N, D, M, K = args.n, 128, args.m, 256
    nchunks = nchunks or args.online
    ring = [torch.from_numpy(synth.sift_like(N, D=D, start=i * N, dtype=np.uint8)).pin_memory() for i in range(4)]
    ctx = hclae.Context(N, D, M, K)
    # dictionaries learned offline on the first chunk (one fresh sweep), weights = that chunk's cluster sizes
    X0 = ring[0].to(dev).float()
    C = torch.zeros((M, K, D), dtype=torch.float32, device=dev)
    codes = torch.zeros((N, M), dtype=torch.uint8, device=dev)
    r = X0.clone()
    ctx.sweep(C, codes, r, 2, init_idx=synth.init_indices(N, M, K), want_err=False)
    n0 = np.stack([np.bincount(codes[:, m].cpu().numpy(), minlength=K) for m in range(M)]).astype(np.int64)
    ctx.online_begin(C, n0)
    del X0
    stage = [torch.empty((N, D), dtype=torch.uint8, device=dev) for _ in range(2)]
    side, main_s = torch.cuda.Stream(), torch.cuda.current_stream()

    def run(count, timed, copy=True):
        copied = [torch.cuda.Event() for _ in range(count)]
        freed = [torch.cuda.Event() for _ in range(count)]
        errs = []
        for i in range(count):
            if copy:
                with torch.cuda.stream(side):
                    if i >= 2:
                        side.wait_event(freed[i - 2])
                    stage[i % 2].copy_(ring[i % 4], non_blocking=True)
                    copied[i].record(side)
                main_s.wait_event(copied[i])
            e = ctx.online_chunk(stage[i % 2], C, codes, r, want_err=(timed and i == count - 1))
            freed[i].record(main_s)
            if e is not None:
                errs.append(e)
        torch.cuda.synchronize()
        return errs

    run(2, False)
    ctx.timing_enable(["assign"])
    t0 = time.perf_counter()
    errs = run(nchunks, True)
    t1 = time.perf_counter()
    ctx.timing_enable([])
    tm = ctx.timing_read()
    a_ms, a_n = tm["assign"]
    # compute alone (chunks already staged) and copy alone, for the overlap figure
    tk = time.perf_counter()
    run(min(nchunks, 8), False, copy=False)
    tk = (time.perf_counter() - tk) / min(nchunks, 8)
    torch.cuda.synchronize()
    tc = time.perf_counter()
    for i in range(4):
        stage[i % 2].copy_(ring[i], non_blocking=True)
    torch.cuda.synchronize()
    tc = (time.perf_counter() - tc) / 4
    per_chunk = (t1 - t0) / nchunks
    flops = 2.0 * N * K * D
    tf = flops / (a_ms / max(a_n, 1) * 1e-3) / 1e12
    ctx.close()
    return {
        "metric": "online DA vectors/sec end to end (uint8 chunks from pinned host memory, D=128, K=256)",
        "value": N / per_chunk, "unit": "vectors/s", "n_gpus": 1, "steps": nchunks, "warmup": 2,
        "ms_per_step": per_chunk * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "online DA: %d of the configuration's 100 chunks of %d SIFT-shaped uint8 vectors (a ring "
                               "of 4 distinct chunks in pinned host memory, reused in turn), M=%d, K=256, one pass per "
                               "chunk (assign, running-sum update, re-assign, residue per stage)" % (nchunks, N, M),
                   "chunks": nchunks, "distinct_chunks": 4,
                   "quant_error_last_chunk": errs[-1] if errs else None},
        "h2d_copy_ms_per_chunk": tc * 1e3, "h2d_GBs": N * D / tc / 1e9,
        "compute_only_ms_per_chunk": tk * 1e3,
        "copy_hidden_fraction": min(1.0, max(0.0, 1.0 - (per_chunk - tk) / tc)),
        "roofline": {"bound": "mfma", "kernel": "k_assign_resident<8>", "achieved": tf, "peak": PEAK_FP32_MFMA_TFLOPS,
                     "unit": "TFLOP/s", "frac": tf / PEAK_FP32_MFMA_TFLOPS, "traffic": None,
                     "avg_launch_ms": a_ms / max(a_n, 1), "launches": a_n},
    }


def m16_bench(args, torch, hclae, synth, dev):
    """128-bit codes (M = 16): the sweep from all-zero dictionaries and the annealing sweep after it, timed once
    each after one untimed pass of both (same states), with E after each of the 32 stages."""
    N, D, M, K, T = args.n, 128, 16, 256, args.iters
    Xg = torch.from_numpy(synth.sift_like(N, D=D)).to(dev)
    idx = synth.init_indices(N, M, K)
    ctx = hclae.Context(N, D, M, K)
    st = State(torch, Xg, M, K)
    st.save("zero")
    res = {}
    for rep in range(2):                                  # the first pass warms up
        st.restore("zero")
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        E1 = ctx.sweep(st.C, st.codes, st.r, T, init_idx=idx)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        E2 = ctx.sweep(st.C, st.codes, st.r, T)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        res = {"fresh_sweep_ms": (t1 - t0) * 1e3, "first_anneal_sweep_ms": (t2 - t1) * 1e3,
               "first_anneal_sweep_value": N * M / (t2 - t1), "unit": "vectors/s per stage",
               "quant_error_per_stage": [float(e) for e in np.concatenate([E1, E2])],
               "note": "N=%d, D=128, M=16, K=256, T=%d; per-stage errors are read back inside the timed calls" % (N, T)}
    ctx.close()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--n", type=int, default=1_000_000)
    ap.add_argument("--m", type=int, default=8)
    ap.add_argument("--iters", type=int, default=10, help="Lloyd iterations T per cool-down")
    ap.add_argument("--queries", type=int, default=10_000)
    ap.add_argument("--shape", choices=["sift", "gist"], default="sift",
                    help="sift: the headline workload (D=128).  gist: the same step on GIST-shaped data (D=960, "
                         "the D-chunked assign kernel), reported beside it, never instead of it")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-breakdown", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="leave out the short runs of the other configurations (GIST shape, 128-bit codes, online "
                         "chunks, multi-path encoding, improved k-means) that the default line carries as extra keys")
    ap.add_argument("--online", type=int, default=0, metavar="CHUNKS",
                    help="instead of the sweep benchmark: stream CHUNKS uint8 chunks of --n vectors from pinned host "
                         "memory through the online learner (ring of 4 distinct chunks) and report end-to-end vectors/s")
    ap.add_argument("--contraction", choices=["f32", "split"], default="f32",
                    help="matrix-core arithmetic of the distance contraction: fp32 MFMA, or fp32 operands split into "
                         "two bf16 terms on the bf16 MFMA (same results; see hclae_set_contraction)")
    ap.add_argument("--no-pruning", action="store_true",
                    help="switch off the exact pruning of the Lloyd iterations (hclae_set_pruning 0): every assignment "
                         "and every centroid sum then runs over all vectors; same results")
    ap.add_argument("--beam", type=int, default=0, metavar="L",
                    help="instead of the sweep benchmark: learn the dictionaries with one fresh sweep, then time the "
                         "multi-path encoder (Sec. 3.3) with L paths over the --n resident vectors")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no sharding, no collectives); use --gpus 1")

    import torch
    from paper_1509_05194_amd import hclae, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    gist = args.shape == "gist"
    if gist and (args.online or args.beam):
        sys.exit("bench.py: --shape gist runs the sweep only")
    if args.online:
        print(json.dumps(online_bench(args, torch, hclae, synth, dev)))
        return
    if args.beam:
        print(json.dumps(beam_bench(args, torch, hclae, synth, dev)))
        return

    extras = not args.no_extras and not gist and not args.no_breakdown
    out = sweep_bench(args, torch, hclae, synth, dev, gist, extras)
    if extras:
        # short runs of the other configurations, each reported as measured under a key of its own
        torch.cuda.empty_cache()
        sub = argparse.Namespace(**vars(args))
        sub.steps, sub.warmup, sub.no_cpu_baseline, sub.no_breakdown = 2, 1, True, True
        sub.m, sub.contraction, sub.no_pruning = 4, "f32", False
        g = sweep_bench(sub, torch, hclae, synth, dev, True, False)
        out["gist_shape"] = {k: g[k] for k in ("value", "unit", "ms_per_step", "steps", "config", "roofline")}
        torch.cuda.empty_cache()
        out["codes_128bit"] = m16_bench(args, torch, hclae, synth, dev)
        torch.cuda.empty_cache()
        sub = argparse.Namespace(**vars(args))
        sub.beam, sub.contraction = 10, "f32"
        b = beam_bench(sub, torch, hclae, synth, dev, steps=1)
        out["multipath_L10"] = {k: b[k] for k in ("value", "unit", "ms_per_step", "steps", "config", "roofline", "kernels")}
        torch.cuda.empty_cache()
        o = online_bench(args, torch, hclae, synth, dev, nchunks=16)
        out["online_chunks"] = {k: o[k] for k in ("value", "unit", "ms_per_step", "steps", "config", "h2d_GBs",
                                                  "compute_only_ms_per_chunk", "copy_hidden_fraction", "roofline")}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
