#!/usr/bin/env python3
"""Benchmark of the per-layer selective-recompute path on one MI355X.

A "step" is one pass of the whole hot path over one synthetic layer:
reposition_keys + score_tokens (issued as the one call ifkv_reposition_score,
which gives the same caches and scores) -> select_topk -> splice_kv ->
recompute_attention, all inputs resident in HBM.  The default workload is the
32K-context Llama-3-8B-shaped layer (64 chunks x 512 tokens in a seeded random
order, 128 prompt tokens) at a recompute ratio of 15 %.

Prints ONE JSON line:
  value      recomputed context tokens per second per layer = k / step time
  roofline   the attention kernel against the bf16 MFMA peak: algorithmic
             flops 4 d H_q sum_r (p_r + 1) per launch over its mean duration,
             measured with HIP events on the stream the kernels run on
  cpu_baseline  the numpy fp64 oracle timed on this machine's host cores on a
             bounded sample of the same workload
  stages     per stage: mean and median time (over repeats of back-to-back
             launches) and achieved algorithmic GB/s or TFLOP/s; for the
             streaming stages also "cold_ms": the same launch rotating over
             five buffer sets, so that nothing it touches is still in a cache
  calibration  what this machine delivers for a plain copy and for a bare MFMA
             loop (constant operands / operands that switch like activations),
             to read the fractions of the published peaks against

`--sweep` runs every BASELINE configuration (C3 at its three ratios) and prints a
markdown table of the stage times instead (the summary kept under profiles/).
Every stage call is marshalled once (Layer.bind) and then re-issued, so the
timed loops contain the C calls and their kernels only.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK = 8.0e12        # B/s, MI355X HBM3E
MFMA_BF16_PEAK = 2.5e15  # flop/s, dense bf16

# HBM bytes per call of the attention stage (attention kernel, plus the combine pass where the launch
# is cut) from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs, scaled by what the same counters read
# for the plain copy kernel: profiles/attn_mfma_kernel_counters_all_configs.md has the commands and
# the raw readings (taken with the kernels as they are now); None for anything else.
ATTENTION_TRAFFIC_BYTES = {("C3", 0.15): 8.662e8, ("C3", 0.05): 3.456e8 + 4.0e7, ("C3", 0.3): 8.399e8,
                           ("C2", 0.15): 8.67e7 + 4.2e7, ("C4", 0.1): 2.003e10, ("C5", 0.15): 1.756e8}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="C3", choices=["C1", "C2", "C3", "C4", "C5"])
    ap.add_argument("--ratio", type=float, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--stage-iters", type=int, default=20, help="launches per timed block of a stage")
    ap.add_argument("--stage-repeats", type=int, default=5, help="timed blocks per stage (median and mean over them)")
    ap.add_argument("--sweep", action="store_true", help="all configurations, markdown table on stdout")
    ap.add_argument("--zero-inputs", action="store_true",
                    help="profiling aid for --only recompute_attention: all-zero K, V and queries (same instruction "
                         "stream, least switching activity: shows how far the clock drops on real data)")
    ap.add_argument("--tune", action="append", default=[], metavar="KEY=VALUE",
                    help="launch-shape knob of include/ifkv_debug.h (sweeps), e.g. attn_split_parts=2")
    ap.add_argument("--only", default=None,
                    choices=["reposition_keys", "score_tokens", "reposition_score", "select_topk", "splice_kv",
                             "recompute_attention", "copy"],
                    help="profiling aid: after set-up run only this stage --stage-iters times and exit")
    return ap.parse_args()


class Bench:
    """One workload set up on the GPU, every stage call marshalled once."""

    def __init__(self, workload, ratio, tune=()):
        import torch

        import paper_2603_05353_amd as pkg
        from workloads import make_recompute_inputs, make_workload, preset
        self.torch = torch
        self.name = workload
        spec = self.spec = preset(workload)
        self.ratio = ratio if ratio is not None else (0.15 if 0.15 in spec.ratios else spec.ratios[0])
        wl = self.wl = make_workload(spec)
        N, M = self.N, self.M = wl.n_ctx, spec.m_prompt
        self.e = 2 if spec.dtype == "bf16" else 4
        dev = "cuda:0"

        def dev_t(x):
            if spec.dtype == "bf16":
                return torch.from_numpy(np.ascontiguousarray(x).view(np.int16)).view(torch.bfloat16).to(dev)
            return torch.from_numpy(np.ascontiguousarray(x)).to(dev)
        self.dev_t = dev_t
        L = self.L = pkg.Layer(spec.dtype, spec.n_q_heads, spec.n_kv_heads, spec.head_dim, spec.rope_theta,
                               max_ctx=N, max_prompt=M)
        for kv in tune:
            key, value = kv.split("=")
            L.set_tuning(key, int(value))
        self.kd = [dev_t(c) for c in wl.k_chunks]
        self.vd = [dev_t(c) for c in wl.v_chunks]
        self.qd = dev_t(wl.q_prompt)
        self.order = wl.chunk_order.tolist()
        self.K, self.V = L.empty_cache(N), L.empty_cache(N)
        self.scores = torch.empty(N, dtype=torch.float32, device=dev)
        k_sel = self.k_sel = L.budget_of(N, self.ratio)     # k = floor(ratio N) as the library evaluates it
        self.idx = torch.empty(max(k_sel, 1), dtype=torch.int32, device=dev)
        # one untimed pass to learn the selected set, then build the recompute rows for it
        L.reposition_keys(self.kd, self.vd, chunk_order=self.order, k_out=self.K, v_out=self.V)
        L.score_tokens(self.K, self.qd, scores=self.scores)
        L.select_topk(self.scores, ratio=self.ratio, idx_out=self.idx)
        torch.cuda.synchronize()
        self.idx_host = self.idx[:k_sel].cpu().numpy().astype(np.int64)
        self.q_sel, self.k_new, self.v_new = make_recompute_inputs(wl, self.idx_host)
        self.q_sel_d, self.k_new_d, self.v_new_d = dev_t(self.q_sel), dev_t(self.k_new), dev_t(self.v_new)
        tdt = torch.bfloat16 if spec.dtype == "bf16" else torch.float32
        self.out = torch.empty(k_sel, spec.n_q_heads, spec.head_dim, dtype=tdt, device=dev)
        self.idx_k = self.idx[:k_sel]
        self.calls = self.bind_calls(self.kd, self.vd, self.K, self.V, self.k_new_d, self.v_new_d)

    def bind_calls(self, kd, vd, K, V, kn, vn):
        L = self.L
        return {
            "reposition_keys": L.bind("reposition_keys", kd, vd, chunk_order=self.order, k_out=K, v_out=V),
            "score_tokens": L.bind("score_tokens", K, self.qd, scores=self.scores),
            "reposition_score": L.bind("reposition_score", kd, vd, self.qd, chunk_order=self.order, k_out=K, v_out=V,
                                       scores=self.scores),
            "select_topk": L.bind("select_topk", self.scores, ratio=self.ratio, idx_out=self.idx),
            "splice_kv": L.bind("splice_kv", kn, vn, self.idx_k, K, V),
            "recompute_attention": L.bind("recompute_attention", self.q_sel_d, self.idx_k, K, V, out=self.out),
        }

    def step(self):
        c = self.calls
        c["reposition_score"]()
        c["select_topk"]()
        c["splice_kv"]()
        c["recompute_attention"]()

    def time_stage(self, fn, iters, repeats):
        """(mean, median) seconds per launch over `repeats` blocks of `iters` back-to-back launches,
        events on the stream the kernels run on."""
        torch = self.torch
        fn()
        torch.cuda.synchronize()
        per = []
        for _ in range(repeats):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(iters):
                fn()
            b.record()
            torch.cuda.synchronize()
            per.append(a.elapsed_time(b) * 1e-3 / iters)
        return float(np.mean(per)), float(np.median(per))

    def stage_times(self, iters, repeats, cold=True):
        torch = self.torch
        t = {name: self.time_stage(fn, iters, repeats) for name, fn in self.calls.items()}
        tc = {}
        if cold:
            # cold-cache variant of the streaming stages: five distinct buffer sets in rotation, so
            # that a launch finds none of its data in the L2s or the 256 MB memory-side cache
            n_sets = 5
            sets = [self.calls]
            for _ in range(n_sets - 1):
                sets.append(self.bind_calls([c.clone() for c in self.kd], [c.clone() for c in self.vd], self.K.clone(),
                                            self.V.clone(), self.k_new_d.clone(), self.v_new_d.clone()))
            turn = [0]

            def rotating(name):
                def call():
                    sets[turn[0] % n_sets][name]()
                    turn[0] += 1
                return call
            for name in ("reposition_keys", "score_tokens", "reposition_score", "splice_kv"):
                tc[name] = self.time_stage(rotating(name), max(iters, 2 * n_sets), repeats)
            del sets
            torch.cuda.empty_cache()
        return t, tc

    def work(self):
        sp, N, M, e, k_sel = self.spec, self.N, self.M, self.e, self.k_sel
        row_bytes = sp.n_kv_heads * sp.head_dim * e
        return {
            "b_repo": 4 * N * row_bytes,                       # K and V, read + write
            "b_score": 2 * N * row_bytes + 4 * N,              # two sweeps over K + the scores
            "b_fused": 5 * N * row_bytes + 4 * N,              # chunks read, caches written, K read once more, scores
            "b_splice": 4 * k_sel * row_bytes + 4 * k_sel,
            "f_score": 2 * 2 * N * M * sp.n_q_heads * sp.head_dim,
            "f_attn": 4.0 * sp.head_dim * sp.n_q_heads * float(np.sum(self.idx_host + 1)),
        }

    def stages_report(self, t, tc):
        w = self.work()

        def entry(name, nbytes=None, flops=None):
            mean, med = t[name]
            d = {"ms": mean * 1e3, "median_ms": med * 1e3}
            if nbytes is not None:
                d["GB/s"] = nbytes / mean / 1e9
                d["frac_hbm"] = nbytes / mean / HBM_PEAK
            if flops is not None:
                d["TFLOP/s"] = flops / mean / 1e12
                d["frac_mfma"] = flops / mean / MFMA_BF16_PEAK
            if name in tc:
                d["cold_ms"] = tc[name][0] * 1e3
            return d
        return {
            "reposition_keys": entry("reposition_keys", w["b_repo"]),
            "score_tokens": entry("score_tokens", w["b_score"], w["f_score"]),
            "reposition_score": entry("reposition_score", w["b_fused"], w["f_score"]),
            "select_topk": dict(entry("select_topk"), launches=1),
            "splice_kv": entry("splice_kv", w["b_splice"]),
            "recompute_attention": entry("recompute_attention", flops=w["f_attn"]),
        }

    def close(self):
        self.L.close()


def run_default(args):
    import torch
    B = Bench(args.workload, args.ratio, args.tune)
    spec, N, M, k_sel, L = B.spec, B.N, B.M, B.k_sel, B.L

    if args.only is not None:
        if args.zero_inputs:
            B.K.zero_(), B.V.zero_(), B.q_sel_d.zero_()
        src = torch.empty(2 * N * spec.n_kv_heads * spec.head_dim * B.e, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        fn = dict(B.calls, copy=lambda: L.copy_bytes(dst, src))[args.only]
        for _ in range(args.stage_iters):
            fn()
        torch.cuda.synchronize()
        print(json.dumps({"only": args.only, "iters": args.stage_iters, "workload": args.workload,
                          "ratio": B.ratio, "copy_bytes": int(src.numel())}))
        B.close()
        return

    for _ in range(args.warmup):
        B.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        B.step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    step_s = (t1 - t0) / args.steps

    t, tc = B.stage_times(args.stage_iters, args.stage_repeats)
    stages = B.stages_report(t, tc)

    # calibration: what a plain copy of the K+V footprint achieves on this machine, and what a bare
    # MFMA loop sustains (about 50 ms per pattern, long enough for the clock to settle)
    row_bytes = spec.n_kv_heads * spec.head_dim * B.e
    src = torch.empty(2 * N * row_bytes, dtype=torch.uint8, device="cuda:0")
    dst = torch.empty_like(src)
    t_copy = B.time_stage(lambda: L.copy_bytes(dst, src), args.stage_iters, args.stage_repeats)[0]
    del src, dst
    sink = torch.empty(L.mfma_probe_sink_floats(), dtype=torch.float32, device="cuda:0")
    probe_iters = 15000
    probe = {}
    for name, pattern in (("constant_operands", 0), ("activation_like_operands", 1)):
        probe_flops = L.mfma_probe(pattern, probe_iters, sink)
        t_p = B.time_stage(lambda: L.mfma_probe(pattern, probe_iters, sink), 3, 1)[0]
        probe[name] = probe_flops / t_p / 1e12

    t_attn = t["recompute_attention"][0]
    f_attn = B.work()["f_attn"]
    t_sum = sum(t[n][0] for n in ("reposition_score", "select_topk", "splice_kv", "recompute_attention"))
    calibration = {
        "copy": {"ms": t_copy * 1e3, "GB/s": 4 * N * row_bytes / t_copy / 1e9},
        "mfma_loop_TFLOP/s": probe,
        "recomputed_tokens_per_s_from_stage_sum": k_sel / t_sum,
        "context_tokens_per_s_from_stage_sum": N / t_sum,
        "recomputed_tokens_per_s_attention_only": k_sel / t_attn,
    }
    if spec.dtype == "bf16":
        roofline = {"kernel": "attn_mfma_kernel", "bound": "mfma", "achieved": f_attn / t_attn / 1e12,
                    "peak": MFMA_BF16_PEAK / 1e12, "unit": "TFLOP/s", "frac": f_attn / t_attn / MFMA_BF16_PEAK,
                    "traffic": ATTENTION_TRAFFIC_BYTES.get((args.workload, B.ratio))}
    else:
        roofline = {"kernel": "attn_generic_kernel", "bound": "alu", "achieved": f_attn / t_attn / 1e12,
                    "peak": 157.3, "unit": "TFLOP/s", "frac": f_attn / t_attn / 157.3e12, "traffic": None}

    result = {
        "metric": "recomputed ctx tokens/s per layer", "value": k_sel / step_s, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": step_s * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": spec.dtype, "data": "synthetic",
        "config": {"workload": f"{args.workload}: {len(B.wl.chunk_len)} chunks, N={N} ctx, M={M} prompt, "
                               f"H_q/H_kv/d={spec.n_q_heads}/{spec.n_kv_heads}/{spec.head_dim}, "
                               f"ratio={B.ratio} (k={k_sel})",
                   "ratio": B.ratio, "n_ctx": N, "k": k_sel},
        "roofline": roofline,
        "stages": stages,
        "calibration": calibration,
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(B.wl, B.ratio, B.q_sel, B.k_new, B.v_new)
    B.close()
    print(json.dumps(result))


def run_sweep(args):
    """Stage times of every BASELINE configuration as a markdown table."""
    import torch
    rows = []
    for name, ratio in (("C2", None), ("C3", 0.05), ("C3", 0.15), ("C3", 0.30), ("C4", None), ("C5", None), ("C1", None)):
        B = Bench(name, ratio, args.tune)
        for _ in range(3):
            B.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(10):
            B.step()
        torch.cuda.synchronize()
        step_ms = (time.perf_counter() - t0) / 10 * 1e3
        t, tc = B.stage_times(args.stage_iters, args.stage_repeats, cold=(name != "C1"))
        st = B.stages_report(t, tc)
        a = st["recompute_attention"]
        frac = a["frac_mfma"] if B.spec.dtype == "bf16" else a["TFLOP/s"] / 157.3

        def us(n, key="ms"):
            return f"{st[n][key] * 1e3:.1f}" if key in st[n] else "-"
        rows.append(f"| {name} | {B.ratio} | {B.N} | {B.k_sel} | {step_ms * 1e3:.0f} | "
                    f"{us('reposition_keys')} / {us('reposition_keys', 'median_ms')} / {us('reposition_keys', 'cold_ms')} ({st['reposition_keys']['frac_hbm']:.2f}) | "
                    f"{us('score_tokens')} / {us('score_tokens', 'median_ms')} / {us('score_tokens', 'cold_ms')} ({st['score_tokens'].get('frac_mfma', 0):.2f}) | "
                    f"{us('reposition_score')} / {us('reposition_score', 'median_ms')} / {us('reposition_score', 'cold_ms')} | "
                    f"{us('select_topk')} / {us('select_topk', 'median_ms')} | "
                    f"{us('splice_kv')} / {us('splice_kv', 'median_ms')} / {us('splice_kv', 'cold_ms')} ({st['splice_kv']['frac_hbm']:.2f}) | "
                    f"{us('recompute_attention')} / {us('recompute_attention', 'median_ms')} | {a['TFLOP/s']:.0f} | {frac:.3f} | "
                    f"{B.k_sel / (step_ms * 1e-3):.3g} |")
        B.close()
        del B
        torch.cuda.empty_cache()
    print("| cfg | ratio | N | k | step us | stage 1: mean / median / cold us (frac HBM) | stage 2: mean / median / cold us (frac MFMA) | "
          "stages 1+2 in one call: mean / median / cold us | stage 3: mean / median us | stage 5: mean / median / cold us (frac HBM) | "
          "stage 4: mean / median us | stage 4 TFLOP/s | stage 4 frac of peak | recomputed tokens/s |")
    print("|" + "---|" * 14)
    print("\n".join(rows))


def main():
    args = parse()
    if args.gpus != 1:
        sys.stderr.write("bench.py: this build runs on one GPU only (--gpus 1); "
                         "no multi-GPU figure is produced.\n")
        sys.exit(2)
    import torch

    import paper_2603_05353_amd as pkg
    if not torch.cuda.is_available():
        sys.stderr.write("bench.py: no GPU visible\n")
        sys.exit(1)
    if not os.path.exists(pkg.LIB_PATH):
        from paper_2603_05353_amd.build import build_library
        build_library()
    if args.sweep:
        run_sweep(args)
    else:
        run_default(args)


def cpu_baseline(wl, ratio, q_sel, k_new, v_new, n_rows_sample=1536):
    """Stages 1, 2, 3, 5 in full; stage 4 on a seeded sample of rows (rows are
    independent), extrapolated by the causal work sum_r (p_r + 1)."""
    from oracle import infoflow_oracle as O
    from workloads import to_f64
    sp = wl.spec
    k64 = [to_f64(c, sp.dtype) for c in wl.k_chunks]
    v64 = [to_f64(c, sp.dtype) for c in wl.v_chunks]
    q64 = to_f64(wl.q_prompt, sp.dtype)
    t = {}
    t0 = time.perf_counter()
    K, V, _, N = O.reposition_keys(k64, v64, wl.chunk_len, wl.chunk_order, sp.rope_theta, sp.pairing)
    t["reposition"] = time.perf_counter() - t0
    t0 = time.perf_counter()
    s = O.score_tokens(K, q64, wl.sm_scale)
    t["score"] = time.perf_counter() - t0
    t0 = time.perf_counter()
    idx = O.select_topk(s, O.budget(N, ratio))
    t["topk"] = time.perf_counter() - t0
    k_sel = len(idx)
    # the benchmark's rows were generated for the GPU's selection of the same size
    qs, kn, vn = (to_f64(x, sp.dtype)[:k_sel] for x in (q_sel, k_new, v_new))
    t0 = time.perf_counter()
    K2, V2 = O.splice_kv(K, V, kn, vn, idx)
    t["splice"] = time.perf_counter() - t0
    g = np.random.Generator(np.random.Philox(key=[sp.seed, 4242]))
    pick = np.sort(g.choice(k_sel, size=min(n_rows_sample, k_sel), replace=False))
    t0 = time.perf_counter()
    O.recompute_attention(qs[pick], idx[pick], K2, V2, wl.sm_scale)
    t_s = time.perf_counter() - t0
    work_all = float(np.sum(idx + 1))
    work_s = float(np.sum(idx[pick] + 1))
    t["attention_extrapolated"] = t_s * work_all / work_s
    total = sum(t.values())
    try:
        import threadpoolctl
        cores = max((p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()), default=os.cpu_count())
    except Exception:
        cores = os.cpu_count()
    return {"value": k_sel / total, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"stages 1,2,3,5 in full; stage 4 on {len(pick)} of {k_sel} selected rows "
                      f"({t_s:.1f} s), scaled by sum(p_r+1) to all rows",
            "seconds": {k: round(v, 3) for k, v in t.items()}, "host_cpus": os.cpu_count()}


if __name__ == "__main__":
    main()
