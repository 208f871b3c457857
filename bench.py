"""Benchmark of the SOCKET decode hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 128k|32k] [--layers 32]

One "step" is one decode step of a Llama-3-8B-shaped attention stack: for each of `layers`
layers (distinct K/V/bucket-id buffers, so the 256 MB Infinity Cache cannot stand in for
HBM) append-hash the new key, soft-hash the query, score every cached key, select the
top-k and run sparse attention over them.  All inputs are synthetic, seeded, and resident
in HBM before the timed region.  The whole step is replayed as one HIP graph.

Prints one JSON line.  Beside the headline (`value`, `roofline`, `cpu_baseline`) it carries:
  paged_b16   the batched configuration: 16 paged sequences of U[8192, 32768] tokens, 64
              consecutive decode steps, each appending one row per sequence
  sweep       hashing + append sweep: 4 x 65536 keys, L in {16,32,64,128} x P in {4,8,10}:
              prefill-hash MFMA utilisation and scoring GB/s per point
  hard_vs_soft  scoring cost of the hard LSH scorer at (P, L) = (2, 300/400/500) beside the
              soft scorer at (10, 60) on a 32K context (the shape of the paper's Table 2)
  hbm_stream_ceiling_gbs  what a kernel that only reads reaches on this GPU
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published

# HBM bytes per launch of the scoring kernel with the select's histogram, 128K workload, from
# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE scaled by a plain copy (profiles/score_kernel_128k.md)
PROFILED_SCORE_TRAFFIC = {("128k", 32, 64, 8): (77.0e6, "profiles/score_kernel_128k.md")}

WORKLOADS = {
    # name: (n, k, seed)   -- the 128K roofline workload and the 32K one
    "128k": (131072, 2048, 1002),
    "32k": (32768, 1024, 1001),
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="128k", choices=sorted(WORKLOADS))
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--L", type=int, default=64, help="hash tables (headline: 64)")
    ap.add_argument("--P", type=int, default=8, help="hyperplanes per table (headline: 8; the paper's main runs: P=10, L=60)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="headline only: skip paged_b16, sweep, hard_vs_soft")
    ap.add_argument("--only", default="", choices=["", "score", "step", "paged", "sweep", "hash"],
                    help="profiling aids: 'score' runs just the scoring kernel (with the select's histogram) "
                         "over all layers, plus a plain 256 MiB copy that calibrates rocprofv3's HBM byte "
                         "counters; 'step' runs the prefill and the timed fused steps and nothing else; "
                         "'paged' / 'sweep' run only that leg; 'hash' only the prefill hash")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--sweep-steps", type=int, default=256)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2602_06283_amd import binding as sk
    from paper_2602_06283_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    stream = torch.cuda.Stream()
    tools = Tools(torch, sk, stream)
    if args.only == "paged":
        with torch.cuda.stream(stream):
            print(json.dumps({"only": "paged", "paged_b16": paged_b16(tools, wl)}))
        return
    if args.only == "sweep":
        with torch.cuda.stream(stream):
            print(json.dumps({"only": "sweep", "sweep": sweep(tools, wl, args.sweep_steps)}))
        return

    n, k, seed = WORKLOADS[args.workload]
    Hq, Hkv, d, L, P, tau = 32, 8, 128, args.L, args.P, 0.5
    NL = args.layers
    extra = args.steps + args.warmup + 64
    n_alloc = (n + extra + 15) // 16 * 16
    id_bytes = sk.codes_bytes(L, P, 16) / 16       # bytes of bucket ids per key and KV head
    timed, capture, ev = tools.timed, tools.capture, tools.ev

    with torch.cuda.stream(stream):
        ctx = sk.Context(sk.make_params(d, Hq, Hkv, L, P, sk.BF16, 1, n_alloc, k))
        layers = []
        for li in range(NL):
            K, V, q, W = wl.device_layer(seed + 100 * li, Hq, Hkv, d, n, n_alloc, L, P)
            codes = torch.zeros((1, Hkv, sk.codes_bytes(L, P, n_alloc)), dtype=torch.uint8, device="cuda")
            layers.append((K, V, q, W, codes))
        scores = torch.zeros((1, Hkv, n_alloc), dtype=torch.float32, device="cuda")
        idx = torch.zeros((1, Hkv, k), dtype=torch.int32, device="cuda")
        nsel = torch.zeros((1, Hkv), dtype=torch.int32, device="cuda")
        out = torch.zeros((NL, 1, Hq, d), dtype=torch.bfloat16, device="cuda")
        zero = torch.zeros(1, dtype=torch.int32, device="cuda")
        one = torch.ones(1, dtype=torch.int32, device="cuda")
        n_t = torch.full((1,), n, dtype=torch.int32, device="cuda")
        pos = torch.full((1,), n, dtype=torch.int32, device="cuda")       # tokens before the append
        length = torch.full((1,), n + 1, dtype=torch.int32, device="cuda")  # tokens after it
        k_t = torch.full((1,), k, dtype=torch.int32, device="cuda")
        stream.synchronize()

        # ---------------- prefill: hash every cached key of every layer (Alg. 1) ----------
        def prefill():
            for (K, V, q, W, codes) in layers:
                ctx.hash_keys(K, W, zero, n_t, 1, n, codes)
        t_prefill_ms = timed(prefill, 2)
        hash_flops = 2.0 * NL * Hkv * n * d * L * P
        hash_bytes = NL * Hkv * n * (d * 2 + id_bytes)
        # the rows that decode steps will append get hashed inside the step
        if args.only == "hash":
            print(json.dumps({"only": "hash", "ms_per_layer": t_prefill_ms / NL,
                              "tflops": hash_flops / (t_prefill_ms * 1e-3) / 1e12}))
            return

        def score_all_binned():
            for (K, V, q, W, codes) in layers:
                ctx.score_keys_binned(codes, length, 1, scores)

        if args.only == "score":
            ctx.soft_hash(layers[0][2], layers[0][3], tau, 1)
            g = capture(score_all_binned)
            us = timed(g.launch, args.steps) * 1e3 / NL
            ctx.reset()
            src = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device="cuda").normal_()
            dst = torch.empty_like(src)
            for _ in range(4):
                dst.copy_(src)           # 256 MiB read + 256 MiB written: counter calibration
            stream.synchronize()
            print(json.dumps({"only": "score", "ctx": n, "layers": NL, "avg_launch_us": us,
                              "algorithmic_bytes": Hkv * (n + 1) * (id_bytes + 4),
                              "gbs": Hkv * (n + 1) * (id_bytes + 4) / (us * 1e-6) / 1e9,
                              "calibration_copy_bytes_each_way": src.numel() * 4}))
            return

        # ---------------- one decode step over all layers --------------------------------
        def step():
            for li, (K, V, q, W, codes) in enumerate(layers):
                ctx.decode_step(q, K, V, codes, W, tau, pos, k_t, 1, 1.0, scores, idx, nsel, out[li])
            pos.add_(1)
            length.add_(1)

        g_step = capture(step)
        for _ in range(args.warmup):
            g_step.launch()
        stream.synchronize()
        t0 = time.perf_counter()
        a, b = ev(), ev()
        a.record(stream)
        for _ in range(args.steps):
            g_step.launch()
        b.record(stream)
        stream.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        ms_per_step = wall_ms / args.steps
        ev_ms_per_step = a.elapsed_time(b) / args.steps
        assert int(nsel.min()) == k and int(length[0]) <= n_alloc
        if args.only == "step":
            print(json.dumps({"only": "step", "ctx": n, "layers": NL, "steps": args.steps,
                              "ms_per_step": ms_per_step, "layer_step_us": ms_per_step * 1e3 / NL}))
            return

        # ---------------- per-stage times: each stage alone, all layers back to back ------
        def stage_graph(body):
            def fn():
                for li, lay in enumerate(layers):
                    body(li, *lay)
            return capture(fn)

        stages = {
            "fused_decode_step": lambda li, K, V, q, W, codes: ctx.decode_step(q, K, V, codes, W, tau, pos, k_t, 1, 1.0,
                                                                          scores, idx, nsel, out[li]),
            "append_hash": lambda li, K, V, q, W, codes: ctx.hash_keys(K, W, pos, one, 1, 1, codes),
            "soft_hash": lambda li, K, V, q, W, codes: ctx.soft_hash(q, W, tau, 1),
            "score": lambda li, K, V, q, W, codes: ctx.score_keys(codes, length, 1, scores),
            "topk": lambda li, K, V, q, W, codes: ctx.topk_select(scores, length, k_t, 1, idx, nsel),
            "sparse_decode": lambda li, K, V, q, W, codes: ctx.sparse_decode(q, K, V, idx, nsel, 1, 1.0, out[li]),
        }
        stage_us = {}
        for name, body in stages.items():
            g = stage_graph(body)
            stage_us[name] = timed(g.launch, 10) * 1e3 / NL     # microseconds per launch
            g.close()
        # the scoring kernel as the fused step runs it: the same pass also builds the select's histogram
        ctx.soft_hash(layers[0][2], layers[0][3], tau, 1)
        g = capture(score_all_binned)
        stage_us["score_with_select_histogram"] = timed(g.launch, 10) * 1e3 / NL
        g.close()
        ctx.reset()
        cur_len = int(length[0])

        # ---------------- what a kernel that only reads reaches (all layers' id buffers) -----
        sink = torch.zeros(1, dtype=torch.int32, device="cuda")

        def read_all():
            for (K, V, q, W, codes) in layers:
                sk.probe_stream_read(codes, sink)
        g = capture(read_all)
        t_read_ms = timed(g.launch, 10)
        g.close()
        stream_gbs = sum(l[4].numel() for l in layers) / (t_read_ms * 1e-3) / 1e9

        # ---------------- how good is the selection?  (evaluation only, layer 0) ------------
        quality = selection_quality(tools, ctx, layers[0], Hq, Hkv, d, k, tau, cur_len, length, k_t, scores, idx, nsel)

        # ---------------- dense attention over the whole context on the same GPU (Eq. 1) ----
        g = stage_graph(lambda li, K, V, q, W, codes: ctx.dense_decode(q, K, V, length, 1, 1.0, out[li]))
        stage_us["dense_decode_baseline"] = timed(g.launch, 5) * 1e3 / NL
        g.close()

        # ---------------- the paper's evaluation protocol on the same step -----------------
        # value-norm weighted ranking (Alg. 3) and 4 sink + 124 local-window tokens always kept
        vns = [torch.empty((1, Hkv, n_alloc), dtype=torch.float32, device="cuda") for _ in layers]
        n_all = torch.full((1,), n_alloc, dtype=torch.int32, device="cuda")

        def norms():
            for (K, V, q, W, codes), vn in zip(layers, vns):
                ctx.value_norms(V, zero, n_all, 1, n_alloc, vn)
        t_norms_ms = timed(norms, 2)
        ctx.set_forced_tokens(4, 124)

        def protocol_step():
            for li, ((K, V, q, W, codes), vn) in enumerate(zip(layers, vns)):
                ctx.decode_step(q, K, V, codes, W, tau, pos, k_t, 1, 1.0, scores, idx, nsel, out[li], vnorm=vn)
        g = capture(protocol_step)
        stage_us["fused_decode_step_value_norms_sink_window"] = timed(g.launch, 10) * 1e3 / NL
        g.close()
        ctx.set_forced_tokens(0, 0)

        cpu = None
        if not args.no_cpu_baseline:
            cpu = cpu_baseline(layers[0], idx.shape[-1], n, Hq, Hkv, d, L, P, tau, NL, args.cpu_seconds)
        del vns, layers, scores, idx, nsel, out
        ctx.close()
        torch.cuda.empty_cache()

        extras = {}
        if not args.no_extras:
            extras["paged_b16"] = paged_b16(tools, wl)
            torch.cuda.empty_cache()
            extras["sweep"] = sweep(tools, wl, args.sweep_steps)
            torch.cuda.empty_cache()
            extras["hard_vs_soft"] = hard_vs_soft(tools, wl)

    # ---------------- roofline of the dominant kernel (scoring) -------------------------
    # algorithmic bytes per launch: every bucket id read once + one fp32 score written per key
    score_bytes = Hkv * cur_len * (id_bytes + 4)
    score_us = stage_us["score_with_select_histogram"]
    score_gbs = score_bytes / (score_us * 1e-6) / 1e9
    chain_bytes = Hkv * (cur_len * (id_bytes + 8) + k * (4 * d + 8))
    chain_us = stage_us["fused_decode_step"]
    traffic, traffic_src = PROFILED_SCORE_TRAFFIC.get((args.workload, NL, L, P), (None, None))

    result = {
        "metric": "decode_steps_per_s",
        "value": 1000.0 / ms_per_step,
        "unit": "steps/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": f"llama3-8b-shaped decode attention, batch 1, ctx {n}, {NL} layers per step "
                        f"(Hq=32, Hkv=8, d=128, bf16 KV, L={L}, P={P}, tau=0.5, top-k={k})",
            "ctx": n, "layers": NL, "L": L, "P": P, "k": k, "graph": "one HIP graph per step",
        },
        "ms_per_step_events": ev_ms_per_step,
        "keys_scored_per_s": Hkv * cur_len / (score_us * 1e-6),
        "layer_step_us": ms_per_step * 1e3 / NL,
        "stage_us_per_layer": stage_us,
        "chain": {"fused_step_us": chain_us, "algorithmic_bytes": chain_bytes,
                  "gbs": chain_bytes / (chain_us * 1e-6) / 1e9,
                  "frac_of_hbm_peak": chain_bytes / (chain_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                  "frac_of_stream_ceiling": chain_bytes / (chain_us * 1e-6) / 1e9 / stream_gbs},
        "roofline": {"kernel": ("score_kernel" if P <= 8 else "score_split_kernel") +
                               ", as socket_decode_step runs it: the pass also builds the select's histogram",
                     "bound": "hbm", "achieved": score_gbs,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": score_gbs / HBM_PEAK_GBS,
                     "traffic": traffic, "traffic_source": traffic_src, "algorithmic_bytes": score_bytes,
                     "avg_launch_us": score_us, "frac_of_stream_ceiling": score_gbs / stream_gbs},
        "hbm_stream_ceiling_gbs": stream_gbs,
        "selection_quality_layer0": quality,
        "dense_baseline": {"us_per_layer": stage_us["dense_decode_baseline"],
                           "gbs": Hkv * cur_len * 4 * d / (stage_us["dense_decode_baseline"] * 1e-6) / 1e9,
                           "sparse_step_speedup": stage_us["dense_decode_baseline"] / stage_us["fused_decode_step"]},
        "value_norms_prefill": {"us_per_layer": t_norms_ms * 1e3 / NL,
                                "gbs": Hkv * n_alloc * (d * 2 + 4) / (t_norms_ms * 1e-3 / NL) / 1e9},
        "hash_prefill": {"ms_per_layer": t_prefill_ms / NL,
                         "tflops": hash_flops / (t_prefill_ms * 1e-3) / 1e12,
                         "mfma_util": hash_flops / (t_prefill_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                         "gbs": hash_bytes / (t_prefill_ms * 1e-3) / 1e9},
    }
    result.update(extras)
    if cpu is not None:
        result["cpu_baseline"] = cpu
    print(json.dumps(result))


class Tools:
    """Event timing and graph capture on one launch stream."""

    def __init__(self, torch, sk, stream):
        self.torch, self.sk, self.stream = torch, sk, stream

    def ev(self):
        return self.torch.cuda.Event(enable_timing=True)

    def timed(self, fn, reps):
        """Mean milliseconds of fn() over reps runs, HIP events on the launch stream."""
        a, b = self.ev(), self.ev()
        fn()
        self.stream.synchronize()
        a.record(self.stream)
        for _ in range(reps):
            fn()
        b.record(self.stream)
        self.stream.synchronize()
        return a.elapsed_time(b) / reps

    def capture(self, fn):
        fn()                      # warm-up outside capture (first-launch work)
        self.stream.synchronize()
        with self.sk.Graph.capture(self.stream) as g:
            fn()
        return g


def selection_quality(tools, ctx, layer0, Hq, Hkv, d, k, tau, cur_len, length, k_t, scores, idx, nsel):
    """Ranking quality of the selection on layer 0 against exact query-key dot products, with
    the metrics of the paper's ranking-quality figure (appendix, metric definitions), computed
    by the CPU oracle: ground-truth relevance of a key = its dot product with the query (mean
    over the G queries that share the KV head), relevant set = the k keys of largest relevance;
    the retrieved list is the selection ordered by the scorer's own score.  Soft scores
    (Alg. 5) beside the hard collision count (Eq. 3, hard form).  Also the share of each query
    head's softmax mass that the selected tokens carry."""
    import numpy as np
    import oracle
    torch, stream = tools.torch, tools.stream
    K0, V0, q0, W0, codes0 = layer0
    G = Hq // Hkv
    Kh = K0[0, :, :cur_len].float().cpu().numpy().astype(np.float64)      # [Hkv, n, d]
    qh = q0[0].float().cpu().numpy().astype(np.float64).reshape(Hkv, G, d)
    logits = np.einsum("hgd,hnd->hgn", qh, Kh)                             # exact dot products
    rel = logits.mean(axis=1)                                              # [Hkv, n]
    res = {}
    for name in ("soft", "hard"):
        if name == "hard":
            ctx.hard_hash(q0, W0, 1)
            ctx.score_keys(codes0, length, 1, scores)
        else:
            ctx.score(q0, codes0, W0, tau, length, 1, scores)
        ctx.topk_select(scores, length, k_t, 1, idx, nsel)
        stream.synchronize()
        sel = idx[0].cpu().numpy()
        sc = scores[0].cpu().numpy()
        prec, jac, ndcg, mass = [], [], [], []
        for h in range(Hkv):
            truth = np.argsort(-rel[h], kind="stable")[:k]
            ranked = sel[h][np.argsort(-sc[h][sel[h]], kind="stable")]    # by the scorer's own score
            prec.append(oracle.precision(sel[h], truth))
            jac.append(oracle.jaccard(sel[h], truth))
            # relevance on the scale of one standard deviation of the head's dot products, so
            # that 2^r stays finite
            unit = rel[h].std()
            ndcg.append(oracle.ndcg(rel[h][ranked] / unit, rel[h] / unit))
            p = np.exp(logits[h] - logits[h].max(axis=1, keepdims=True))
            p /= p.sum(axis=1, keepdims=True)
            mass.append(float(p[:, sel[h]].sum(axis=1).mean()))
        res[name] = {"precision": float(np.mean(prec)), "jaccard": float(np.mean(jac)), "ndcg": float(np.mean(ndcg)),
                     "softmax_mass_kept": float(np.mean(mass))}
    res["metrics_by"] = "oracle (CPU): precision, jaccard, ndcg of the appendix's metric definitions"
    return res


def paged_b16(tools, wl, B=16, steps=64, NL=8, seed=1003):
    """The batched configuration: B paged sequences of U[8192, 32768] tokens (16-token blocks,
    random block table), L = 64, P = 8, k = max(256, 2 % of the length); `steps` consecutive
    fused decode steps over NL layers of distinct buffers (one HIP graph per step), each step
    appending one key/value row per sequence and taking new queries."""
    import numpy as np
    torch, sk, stream = tools.torch, tools.sk, tools.stream
    Hq, Hkv, d, L, P, page, tau = 32, 8, 128, 64, 8, 16, 0.5
    lens, _ = wl.config_batched_lengths(seed, B)
    warm = 2
    cap = (int(lens.max()) + steps + warm + page - 1) // page * page
    kk = np.maximum(256, np.ceil(0.02 * (lens + steps))).astype(np.int32)
    max_k = int(kk.max())
    table, nblocks = wl.make_block_table(seed, np.full(B, cap), page)
    ctx = sk.Context(sk.make_params(d, Hq, Hkv, L, P, sk.BF16, B, cap, max_k, page_size=page,
                                    max_blocks_per_seq=table.shape[1], num_blocks=nblocks))
    bt = torch.from_numpy(table).cuda()
    len_t = torch.from_numpy(lens).cuda()
    zero = torch.zeros(B, dtype=torch.int32, device="cuda")
    layers = []
    for li in range(NL):
        K, V, qs, W = wl.device_paged_layer(seed + 100 * li, B, Hq, Hkv, d, lens, cap, page, table, nblocks, L, P,
                                            steps + warm)
        codes = torch.zeros((nblocks, Hkv, sk.codes_bytes(L, P, page)), dtype=torch.uint8, device="cuda")
        ctx.hash_keys(K, W, zero, len_t, B, int(lens.max()), codes, block_table=bt)
        layers.append((K, V, qs, W, codes, torch.empty((B, Hq, d), dtype=torch.bfloat16, device="cuda")))
    scores = torch.zeros((B, Hkv, cap), dtype=torch.float32, device="cuda")
    idx = torch.zeros((B, Hkv, max_k), dtype=torch.int32, device="cuda")
    nsel = torch.zeros((B, Hkv), dtype=torch.int32, device="cuda")
    out = torch.zeros((NL, B, Hq, d), dtype=torch.bfloat16, device="cuda")
    pos = len_t.clone()
    k_t = torch.from_numpy(kk).cuda()

    def new_queries(s):
        for lay in layers:
            lay[5].copy_(lay[2][s])

    def step():
        for li, (K, V, qs, W, codes, q) in enumerate(layers):
            ctx.decode_step(q, K, V, codes, W, tau, pos, k_t, B, 1.0, scores, idx, nsel, out[li], block_table=bt)
        pos.add_(1)
    new_queries(0)
    g = tools.capture(step)          # (its warm-up call is decode step 0)
    new_queries(1)
    g.launch()
    stream.synchronize()
    a, b = tools.ev(), tools.ev()
    a.record(stream)
    for s in range(steps):
        new_queries(warm + s)
        g.launch()
    b.record(stream)
    stream.synchronize()
    us = a.elapsed_time(b) / steps / NL * 1e3
    ok = bool((nsel.cpu().numpy() == kk[:, None]).all())
    g.close()
    # the two largest kernels of the step on their own (same buffers, final lengths)
    cur = pos.clone()

    def only(body):
        def fn():
            for lay in layers:
                body(*lay)
        g2 = tools.capture(fn)
        t = tools.timed(g2.launch, 5) * 1e3 / NL
        g2.close()
        return t
    us_score = only(lambda K, V, qs, W, codes, q: ctx.score_keys(codes, cur, B, scores, block_table=bt))
    us_soft = only(lambda K, V, qs, W, codes, q: ctx.soft_hash(q, W, tau, B))
    tot = int(lens.sum()) + B * (warm + steps // 2)          # tokens scored per layer-step, mid-run
    id_bytes = sk.codes_bytes(L, P, 16) / 16
    chain_bytes = Hkv * (tot * (id_bytes + 8) + int(kk.sum()) * (4 * d + 8))
    ctx.close()
    return {"workload": f"batch {B}, paged (16-token blocks, random table), lengths U[8192,32768] (sum {int(lens.sum())}), "
                        f"L=64, P=8, k=max(256, 2%) = {int(kk.min())}..{int(kk.max())}, {steps} appending steps, {NL} layers",
            "us_per_layer_step": us, "sequence_layer_steps_per_s": B / (us * 1e-6),
            "keys_scored_per_s": Hkv * tot / (us * 1e-6), "selected_counts_ok": ok,
            "chain": {"algorithmic_bytes": chain_bytes, "gbs": chain_bytes / (us * 1e-6) / 1e9,
                      "frac_of_hbm_peak": chain_bytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS},
            "score_us": us_score, "score_gbs": Hkv * (tot + B * steps // 2) * (id_bytes + 4) / (us_score * 1e-6) / 1e9,
            "soft_hash_us": us_soft}


def sweep(tools, wl, steps=256, B=4, n=65536, seed=1004):
    """Hashing and append sweep: B x n keys, 8 KV heads, d = 128, bf16; for every (L, P) in
    {16,32,64,128} x {4,8,10}: prefill hash of the whole cache (MFMA utilisation), then `steps`
    fused decode steps, each appending and hashing one key per sequence, scoring every key and
    selecting k = 1024; the scoring kernel alone for its GB/s.  Small id buffers are replicated
    (distinct W, distinct ids) until they exceed the 256 MB Infinity Cache."""
    import numpy as np
    torch, sk, stream = tools.torch, tools.sk, tools.stream
    Hq, Hkv, d, k, tau = 32, 8, 128, 1024, 0.5
    cap = (n + steps + 32 + 15) // 16 * 16
    K, V, q = wl.device_batch(seed, B, Hq, Hkv, d, n, cap)
    zero = torch.zeros(B, dtype=torch.int32, device="cuda")
    n_t = torch.full((B,), n, dtype=torch.int32, device="cuda")
    k_t = torch.full((B,), k, dtype=torch.int32, device="cuda")
    scores = torch.zeros((B, Hkv, cap), dtype=torch.float32, device="cuda")
    idx = torch.zeros((B, Hkv, k), dtype=torch.int32, device="cuda")
    nsel = torch.zeros((B, Hkv), dtype=torch.int32, device="cuda")
    out = torch.zeros((B, Hq, d), dtype=torch.bfloat16, device="cuda")
    points = []
    for P in (4, 8, 10):
        for L in (16, 32, 64, 128):
            ctx = sk.Context(sk.make_params(d, Hq, Hkv, L, P, sk.BF16, B, cap, k))
            per_copy = B * Hkv * sk.codes_bytes(L, P, cap)
            copies = int(min(16, max(2, -(-600_000_000 // per_copy))))
            gen = torch.Generator(device="cuda")
            gen.manual_seed(seed + 7 * L + P)
            Ws = [torch.randn((Hkv, d, L * P), generator=gen, device="cuda").to(torch.bfloat16) for _ in range(copies)]
            cs = [torch.zeros((B, Hkv, sk.codes_bytes(L, P, cap)), dtype=torch.uint8, device="cuda") for _ in range(copies)]

            def prefill():
                for W, c in zip(Ws, cs):
                    ctx.hash_keys(K, W, zero, n_t, B, n, c)
            t_hash = tools.timed(prefill, 2) / copies                      # ms per cache
            flops = 2.0 * B * Hkv * n * d * L * P
            pos = n_t.clone()

            def step():
                for W, c in zip(Ws, cs):
                    ctx.decode_step(q, K, V, c, W, tau, pos, k_t, B, 1.0, scores, idx, nsel, out)
                pos.add_(1)
            g = tools.capture(step)
            a, b = tools.ev(), tools.ev()
            a.record(stream)
            for _ in range(steps):
                g.launch()
            b.record(stream)
            stream.synchronize()
            step_us = a.elapsed_time(b) / steps / copies * 1e3
            ok = bool((nsel == k).all())
            g.close()
            cur = pos.clone()

            def score_all():
                for c in cs:
                    ctx.score_keys(c, cur, B, scores)
            g = tools.capture(score_all)
            # (median of five batches of five launches: a single short batch right after the
            # decode loop read up to 50 % high now and then)
            score_us = sorted(tools.timed(g.launch, 5) for _ in range(5))[2] / copies * 1e3
            g.close()
            id_bytes = sk.codes_bytes(L, P, 16) / 16
            sbytes = B * Hkv * int(cur[0]) * (id_bytes + 4)
            points.append({"L": L, "P": P, "id_bytes_per_key": id_bytes, "copies": copies,
                           "hash_ms": t_hash, "hash_tflops": flops / (t_hash * 1e-3) / 1e12,
                           "hash_mfma_util": flops / (t_hash * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                           "decode_step_us": step_us, "steps": steps, "selected_counts_ok": ok,
                           "score_us": score_us, "score_gbs": sbytes / (score_us * 1e-6) / 1e9,
                           "score_frac_of_hbm_peak": sbytes / (score_us * 1e-6) / 1e9 / HBM_PEAK_GBS})
            ctx.close()
            del Ws, cs
            torch.cuda.empty_cache()
    return {"workload": f"batch {B}, 8 KV heads, d=128, n={n}, bf16, k=1024, {steps} decode steps per point", "points": points}


def hard_vs_soft(tools, wl, n=32768, seed=1001):
    """Scoring cost of the hard LSH scorer (Eq. 3, hard form) at (P, L) = (2, 300/400/500) beside
    the soft scorer at the paper's main setting (10, 60), one sequence of 32768 keys, 8 KV heads:
    the paper's cost table has many 2-plane tables cost 2.7-4.2x what 60 ten-plane ones cost.
    Here four 2-bit ids share a byte and a byte's look-up returns the sum of its four tables'
    terms, so (2, 300..500) reads 128 bytes per key (two chunks of 64 bytes) against 80 at
    (10, 60).  Each point: caches of distinct ids so that HBM is what is read."""
    torch, sk, stream = tools.torch, tools.sk, tools.stream
    Hq, Hkv, d = 32, 8, 128
    cap = n + 16
    K, V, q = wl.device_batch(seed, 1, Hq, Hkv, d, n, cap)
    zero = torch.zeros(1, dtype=torch.int32, device="cuda")
    n_t = torch.full((1,), n, dtype=torch.int32, device="cuda")
    scores = torch.zeros((1, Hkv, cap), dtype=torch.float32, device="cuda")
    rows = []
    for (P, L, hard) in ((10, 60, False), (2, 300, True), (2, 400, True), (2, 500, True)):
        ctx = sk.Context(sk.make_params(d, Hq, Hkv, L, P, sk.BF16, 1, cap, 1024))
        per_copy = Hkv * sk.codes_bytes(L, P, cap)
        copies = int(min(32, max(2, -(-600_000_000 // per_copy))))
        gen = torch.Generator(device="cuda")
        gen.manual_seed(seed + 11 * L + P)
        Ws = [torch.randn((Hkv, d, L * P), generator=gen, device="cuda").to(torch.bfloat16) for _ in range(copies)]
        cs = [torch.zeros((1, Hkv, sk.codes_bytes(L, P, cap)), dtype=torch.uint8, device="cuda") for _ in range(copies)]
        for W, c in zip(Ws, cs):
            ctx.hash_keys(K, W, zero, n_t, 1, n, c)
        if hard:
            ctx.hard_hash(q, Ws[0], 1)
        else:
            ctx.soft_hash(q, Ws[0], 0.5, 1)

        def score_all():
            for c in cs:
                ctx.score_keys(c, n_t, 1, scores)
        g = tools.capture(score_all)
        us = tools.timed(g.launch, 10) / copies * 1e3
        g.close()
        id_bytes = sk.codes_bytes(L, P, 16) / 16
        rows.append({"scorer": "hard" if hard else "soft", "P": P, "L": L, "id_bits_per_key": id_bytes * 8,
                     "paper_bits_per_key": P * L, "score_us": us,
                     "gbs": Hkv * n * (id_bytes + 4) / (us * 1e-6) / 1e9})
        ctx.close()
        del Ws, cs
        torch.cuda.empty_cache()
    base = rows[0]["score_us"]
    for r in rows:
        r["time_vs_soft_10_60"] = r["score_us"] / base
    return {"workload": f"batch 1, 8 KV heads, n={n}", "rows": rows,
            "paper_context": "the paper's cost table (another GPU, its own kernel): 0.387 ms at (10,60); hard LSH "
                             "1.027 / 1.328 / 1.629 ms at (2,300) / (2,400) / (2,500) = 2.65x / 3.43x / 4.20x"}


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(layer0, k, n, Hq, Hkv, d, L, P, tau, NL, budget_s):
    """The CPU oracle, as it stands, on one layer's share of a decode step (all 8 KV heads of
    layer 0: hash the appended key, soft-hash 4 queries per head, score n keys, full-sort
    top-k, attention over the k rows), repeated for about `budget_s` seconds; wall seconds per
    stage are kept apart."""
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    import numpy as np
    import harness as hz
    import oracle

    K, V, q, W, codes = layer0
    Kh = K[0, :, :n + 1].float().cpu().numpy()
    Vh = V[0, :, :n + 1].float().cpu().numpy()
    qh = q[0].float().cpu().numpy()
    Wh = W.float().cpu().numpy()
    rows = hz.rows_from_device(codes.view(1, Hkv, -1, hz.lpad_of(L, P) * (1 if P <= 8 else 2)) if not hz.packed(P)
                               else codes.view(1, Hkv, -1, 20 * hz.lpad_of(L)), L, P)
    nat = hz.codes_to_natural(rows[0, :, :n + 1], L, P=P).astype(np.uint16)
    G = Hq // Hkv
    stage = {"hash_appended_key": 0.0, "soft_probs": 0.0, "score": 0.0, "topk": 0.0, "attention": 0.0}
    clock = time.perf_counter

    def layer_step(record):
        for h in range(Hkv):
            t0 = clock()
            new_code, _ = oracle.hash_keys(Kh[h, n:n + 1], Wh[h], L, P)
            c = nat[h]
            c[n] = new_code[0]
            t1 = clock()
            p = np.stack([oracle.soft_probs(qh[h * G + g], Wh[h], L, P, tau) for g in range(G)])
            t2 = clock()
            s = oracle.score(c, p, P)
            t3 = clock()
            sel, cnt = oracle.topk(s, k)
            t4 = clock()
            for g in range(G):
                oracle.sparse_decode(qh[h * G + g], Kh[h], Vh[h], sel[:cnt], 1.0)
            t5 = clock()
            if record:
                for name, dt in zip(stage, (t1 - t0, t2 - t1, t3 - t2, t4 - t3, t5 - t4)):
                    stage[name] += dt

    layer_step(False)
    reps, t0 = 0, clock()
    while True:
        layer_step(True)
        reps += 1
        el = clock() - t0
        if el >= budget_s or reps >= 200:
            break
    per_layer = el / reps
    return {"value": 1.0 / (per_layer * NL), "unit": "steps/s", "cores": oracle.num_threads(),
            "kind": "oracle", "cpu_model": cpu_model(),
            "stage_seconds_per_layer_step": {name: t / reps for name, t in stage.items()},
            "sample": f"{reps} layer-steps of layer 0 (8 KV heads, ctx {n}) in {el:.1f} s; "
                      f"a decode step is {NL} layer-steps, so value = 1/({NL} x {per_layer:.3f} s); "
                      f"only the scoring loop is multi-threaded in the oracle"}


if __name__ == "__main__":
    main()
