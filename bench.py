#!/usr/bin/env python3
"""Benchmark of the per-layer selective-recompute path on one MI355X.

A "step" is one pass of the whole hot path over one synthetic layer:
reposition_keys -> score_tokens -> select_topk -> splice_kv ->
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
  stages     per-stage mean time and achieved algorithmic GB/s or TFLOP/s; for
             the streaming stages also "cold_ms": the same launch rotating over
             five buffer sets, so that nothing it touches is still in a cache
  calibration  what this machine delivers for a plain copy and for a bare MFMA
             loop (constant operands / operands that switch like activations),
             to read the fractions of the published peaks against
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

# HBM bytes per attention launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# runs, scaled by what the same counters read for the plain copy kernel
# (profiles/attn_mfma_kernel_C3_ratio015_counters.md); None for workloads that
# were not profiled.
ATTENTION_TRAFFIC_BYTES = {("C3", 0.15): 8.568e8}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="C3", choices=["C1", "C2", "C3", "C4", "C5"])
    ap.add_argument("--ratio", type=float, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--stage-iters", type=int, default=30)
    ap.add_argument("--zero-inputs", action="store_true",
                    help="profiling aid for --only recompute_attention: all-zero K, V and queries (same instruction "
                         "stream, least switching activity: shows how far the clock drops on real data)")
    ap.add_argument("--tune", action="append", default=[], metavar="KEY=VALUE",
                    help="launch-shape knob of include/ifkv_debug.h (sweeps), e.g. attn_wg_per_head=48")
    ap.add_argument("--only", default=None,
                    choices=["reposition_keys", "score_tokens", "select_topk", "splice_kv",
                             "recompute_attention", "copy"],
                    help="profiling aid: after set-up run only this stage --stage-iters times and exit")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        sys.stderr.write("bench.py: this build runs on one GPU only (--gpus 1); "
                         "no multi-GPU figure is produced.\n")
        sys.exit(2)

    import torch

    import paper_2603_05353_amd as pkg
    from workloads import make_recompute_inputs, make_workload, preset, to_f64

    if not torch.cuda.is_available():
        sys.stderr.write("bench.py: no GPU visible\n")
        sys.exit(1)
    if not os.path.exists(pkg.LIB_PATH):
        from paper_2603_05353_amd.build import build_library
        build_library()

    dev = "cuda:0"
    spec = preset(args.workload)
    ratio = args.ratio if args.ratio is not None else (0.15 if 0.15 in spec.ratios else spec.ratios[0])
    wl = make_workload(spec)
    N, M = wl.n_ctx, spec.m_prompt
    e = 2 if spec.dtype == "bf16" else 4
    tdt = torch.bfloat16 if spec.dtype == "bf16" else torch.float32

    def dev_t(x):
        if spec.dtype == "bf16":
            return torch.from_numpy(np.ascontiguousarray(x).view(np.int16)).view(torch.bfloat16).to(dev)
        return torch.from_numpy(np.ascontiguousarray(x)).to(dev)

    L = pkg.Layer(spec.dtype, spec.n_q_heads, spec.n_kv_heads, spec.head_dim, spec.rope_theta,
                  max_ctx=N, max_prompt=M)
    for kv in args.tune:
        key, value = kv.split("=")
        L.set_tuning(key, int(value))
    kd = [dev_t(c) for c in wl.k_chunks]
    vd = [dev_t(c) for c in wl.v_chunks]
    qd = dev_t(wl.q_prompt)
    order = wl.chunk_order.tolist()
    K = torch.empty(N, spec.n_kv_heads, spec.head_dim, dtype=tdt, device=dev)
    V = torch.empty_like(K)
    scores = torch.empty(N, dtype=torch.float32, device=dev)
    k_sel = L.budget_of(N, ratio)     # k = floor(ratio N) as the library evaluates it (host only)
    idx = torch.empty(max(k_sel, 1), dtype=torch.int32, device=dev)

    # one untimed pass to learn the selected set, then build the recompute rows for it
    L.reposition_keys(kd, vd, chunk_order=order, k_out=K, v_out=V)
    L.score_tokens(K, qd, scores=scores)
    L.select_topk(scores, ratio=ratio, idx_out=idx)
    torch.cuda.synchronize()
    idx_host = idx[:k_sel].cpu().numpy().astype(np.int64)
    q_sel, k_new, v_new = make_recompute_inputs(wl, idx_host)
    q_sel_d, k_new_d, v_new_d = dev_t(q_sel), dev_t(k_new), dev_t(v_new)
    out = torch.empty(k_sel, spec.n_q_heads, spec.head_dim, dtype=tdt, device=dev)
    idx_k = idx[:k_sel]

    if args.only is not None:
        if args.zero_inputs:
            K.zero_(), V.zero_(), q_sel_d.zero_()
        src = torch.empty(2 * N * spec.n_kv_heads * spec.head_dim * e, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        fn = {
            "reposition_keys": lambda: L.reposition_keys(kd, vd, chunk_order=order, k_out=K, v_out=V),
            "score_tokens": lambda: L.score_tokens(K, qd, scores=scores),
            "select_topk": lambda: L.select_topk(scores, ratio=ratio, idx_out=idx),
            "splice_kv": lambda: L.splice_kv(k_new_d, v_new_d, idx_k, K, V),
            "recompute_attention": lambda: L.recompute_attention(q_sel_d, idx_k, K, V, out=out),
            "copy": lambda: L.copy_bytes(dst, src),
        }[args.only]
        for _ in range(args.stage_iters):
            fn()
        torch.cuda.synchronize()
        print(json.dumps({"only": args.only, "iters": args.stage_iters, "workload": args.workload,
                          "ratio": ratio, "copy_bytes": int(src.numel())}))
        L.close()
        return

    def step():
        L.reposition_keys(kd, vd, chunk_order=order, k_out=K, v_out=V)
        L.score_tokens(K, qd, scores=scores)
        L.select_topk(scores, ratio=ratio, idx_out=idx)
        L.splice_kv(k_new_d, v_new_d, idx_k, K, V)
        L.recompute_attention(q_sel_d, idx_k, K, V, out=out)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    step_s = (t1 - t0) / args.steps

    # ---- per-stage timing with events on the kernels' stream ----------------------
    def time_stage(fn, iters):
        fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(iters):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e-3 / iters

    it = args.stage_iters
    t_repo = time_stage(lambda: L.reposition_keys(kd, vd, chunk_order=order, k_out=K, v_out=V), it)
    t_score = time_stage(lambda: L.score_tokens(K, qd, scores=scores), it)
    t_topk = time_stage(lambda: L.select_topk(scores, ratio=ratio, idx_out=idx), it)
    t_splice = time_stage(lambda: L.splice_kv(k_new_d, v_new_d, idx_k, K, V), it)
    t_attn = time_stage(lambda: L.recompute_attention(q_sel_d, idx_k, K, V, out=out), it)

    # cold-cache variant of the streaming stages: five distinct buffer sets in rotation, so
    # that a launch finds none of its data in the L2s or the 256 MB memory-side cache
    n_sets = 5
    kd_sets = [kd] + [[c.clone() for c in kd] for _ in range(n_sets - 1)]
    vd_sets = [vd] + [[c.clone() for c in vd] for _ in range(n_sets - 1)]
    K_sets = [K] + [K.clone() for _ in range(n_sets - 1)]
    V_sets = [V] + [V.clone() for _ in range(n_sets - 1)]
    kn_sets = [k_new_d] + [k_new_d.clone() for _ in range(n_sets - 1)]
    vn_sets = [v_new_d] + [v_new_d.clone() for _ in range(n_sets - 1)]
    turn = [0]

    def rotating(fn):
        def call():
            i = turn[0] % n_sets
            turn[0] += 1
            fn(i)
        return call

    it_cold = max(it, 2 * n_sets)
    tc_repo = time_stage(rotating(lambda i: L.reposition_keys(kd_sets[i], vd_sets[i], chunk_order=order,
                                                              k_out=K_sets[i], v_out=V_sets[i])), it_cold)
    tc_score = time_stage(rotating(lambda i: L.score_tokens(K_sets[i], qd, scores=scores)), it_cold)
    tc_splice = time_stage(rotating(lambda i: L.splice_kv(kn_sets[i], vn_sets[i], idx_k, K_sets[i], V_sets[i])), it_cold)
    del kd_sets, vd_sets, K_sets, V_sets, kn_sets, vn_sets

    # calibration: what a plain copy of the K+V footprint achieves on this machine, and what a bare
    # MFMA loop sustains (about 50 ms per pattern, long enough for the clock to settle)
    src = torch.empty(2 * N * spec.n_kv_heads * spec.head_dim * e, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    t_copy = time_stage(lambda: L.copy_bytes(dst, src), it)
    del src, dst
    sink = torch.empty(L.mfma_probe_sink_floats(), dtype=torch.float32, device=dev)
    probe_iters = 15000
    probe = {}
    for name, pattern in (("constant_operands", 0), ("activation_like_operands", 1)):
        probe_flops = L.mfma_probe(pattern, probe_iters, sink)
        t_p = time_stage(lambda: L.mfma_probe(pattern, probe_iters, sink), 3)
        probe[name] = probe_flops / t_p / 1e12

    row_bytes = spec.n_kv_heads * spec.head_dim * e
    b_repo = 4 * N * row_bytes                       # K and V, read + write
    b_score = 2 * N * row_bytes + 4 * N              # two sweeps over K + the scores
    b_splice = 4 * k_sel * row_bytes + 4 * k_sel
    f_score = 2 * 2 * N * M * spec.n_q_heads * spec.head_dim
    f_attn = 4.0 * spec.head_dim * spec.n_q_heads * float(np.sum(idx_host + 1))
    stages = {
        "reposition_keys": {"ms": t_repo * 1e3, "GB/s": b_repo / t_repo / 1e9, "frac_hbm": b_repo / t_repo / HBM_PEAK},
        "score_tokens": {"ms": t_score * 1e3, "GB/s": b_score / t_score / 1e9, "frac_hbm": b_score / t_score / HBM_PEAK,
                         "TFLOP/s": f_score / t_score / 1e12, "frac_mfma": f_score / t_score / MFMA_BF16_PEAK},
        "select_topk": {"ms": t_topk * 1e3, "launches": 1},
        "splice_kv": {"ms": t_splice * 1e3, "GB/s": b_splice / t_splice / 1e9, "frac_hbm": b_splice / t_splice / HBM_PEAK},
        "recompute_attention": {"ms": t_attn * 1e3, "TFLOP/s": f_attn / t_attn / 1e12,
                                "frac_mfma": f_attn / t_attn / MFMA_BF16_PEAK},
    }
    stages["reposition_keys"]["cold_ms"] = tc_repo * 1e3
    stages["score_tokens"]["cold_ms"] = tc_score * 1e3
    stages["splice_kv"]["cold_ms"] = tc_splice * 1e3
    t_sum = t_repo + t_score + t_topk + t_splice + t_attn
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
                    "traffic": ATTENTION_TRAFFIC_BYTES.get((args.workload, ratio))}
    else:
        roofline = {"kernel": "attn_generic_kernel", "bound": "alu", "achieved": f_attn / t_attn / 1e12,
                    "peak": 157.3, "unit": "TFLOP/s", "frac": f_attn / t_attn / 157.3e12, "traffic": None}

    result = {
        "metric": "recomputed ctx tokens/s per layer", "value": k_sel / step_s, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": step_s * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": spec.dtype, "data": "synthetic",
        "config": {"workload": f"{args.workload}: {len(wl.chunk_len)} chunks, N={N} ctx, M={M} prompt, "
                               f"H_q/H_kv/d={spec.n_q_heads}/{spec.n_kv_heads}/{spec.head_dim}, "
                               f"ratio={ratio} (k={k_sel})",
                   "ratio": ratio, "n_ctx": N, "k": k_sel},
        "roofline": roofline,
        "stages": stages,
        "calibration": calibration,
    }

    # ---- the oracle on the host cores, bounded sample --------------------------------
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, ratio, q_sel, k_new, v_new)
    L.close()
    print(json.dumps(result))


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
