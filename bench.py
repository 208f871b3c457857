"""Benchmark of the SOCKET decode hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 128k|32k] [--layers 32]

One "step" is one decode step of a Llama-3-8B-shaped attention stack: for each of `layers`
layers (distinct K/V/bucket-id buffers, so the 256 MB Infinity Cache cannot stand in for
HBM) append-hash the new key, soft-hash the query, score every cached key, select the
top-k and run sparse attention over them.  All inputs are synthetic, seeded, and resident
in HBM before the timed region.  The whole step is replayed as one HIP graph.

Prints one JSON line (see the keys at the bottom).
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

MEASURED_SCORE_TRAFFIC = {("128k", 32): 73876 * 1024}   # bytes per score_kernel launch

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
    ap.add_argument("--only", default="", choices=["", "score", "step"],
                    help="profiling aids: 'score' runs just the scoring kernel over all layers "
                         "(plus a plain 256 MiB copy that calibrates rocprofv3's HBM byte counters); "
                         "'step' runs the prefill and the timed fused steps and nothing else, so a "
                         "kernel trace holds the step's own kernels only")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
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
    n, k, seed = WORKLOADS[args.workload]
    Hq, Hkv, d, L, P, tau = 32, 8, 128, args.L, args.P, 0.5
    NL = args.layers
    extra = args.steps + args.warmup + 64
    n_alloc = (n + extra + 15) // 16 * 16
    id_bytes = sk.codes_bytes(L, P, 16) / 16       # bytes of bucket ids per key and KV head

    stream = torch.cuda.Stream()
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

        def ev():
            return torch.cuda.Event(enable_timing=True)

        def timed(fn, reps):
            """Mean milliseconds of fn() over reps runs, HIP events on the launch stream."""
            a, b = ev(), ev()
            fn()
            stream.synchronize()
            a.record(stream)
            for _ in range(reps):
                fn()
            b.record(stream)
            stream.synchronize()
            return a.elapsed_time(b) / reps

        def capture(fn):
            fn()                      # warm-up outside capture (first-launch work)
            stream.synchronize()
            with sk.Graph.capture(stream) as g:
                fn()
            return g

        # ---------------- prefill: hash every cached key of every layer (Alg. 1) ----------
        def prefill():
            for (K, V, q, W, codes) in layers:
                ctx.hash_keys(K, W, zero, n_t, 1, n, codes)
        t_prefill_ms = timed(prefill, 2)
        hash_flops = 2.0 * NL * Hkv * n * d * L * P
        hash_bytes = NL * Hkv * n * (d * 2 + id_bytes)
        # the rows that decode steps will append get hashed inside the step

        if args.only == "score":
            ctx.soft_hash(layers[0][2], layers[0][3], tau, 1)

            def score_all():
                for (K, V, q, W, codes) in layers:
                    ctx.score_keys(codes, n_t, 1, scores)
            g = capture(score_all)
            us = timed(g.launch, args.steps) * 1e3 / NL
            src = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device="cuda").normal_()
            dst = torch.empty_like(src)
            for _ in range(4):
                dst.copy_(src)           # 256 MiB read + 256 MiB written: counter calibration
            stream.synchronize()
            print(json.dumps({"only": "score", "ctx": n, "layers": NL, "avg_launch_us": us,
                              "algorithmic_bytes": Hkv * n * (id_bytes + 4),
                              "gbs": Hkv * n * (id_bytes + 4) / (us * 1e-6) / 1e9,
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
        # the same step with the selection ordered before the attention (bit-repeatable output)
        ctx.set_deterministic(True)
        g = stage_graph(stages["fused_decode_step"])
        stage_us["fused_decode_step_deterministic"] = timed(g.launch, 10) * 1e3 / NL
        g.close()
        ctx.set_deterministic(False)
        cur_len = int(length[0])

        # ---------------- how good is the selection?  (evaluation only, layer 0) ------------
        # Against exact q.k on the same synthetic layer: share of each query head's softmax
        # mass that the selected tokens carry, and precision of the selected set against the
        # exact top-k of the group-mean logit.  Soft scores vs the hard collision count (Eq. 3).
        def selection_quality(hard):
            K0, V0, q0, W0, codes0 = layers[0]
            if hard:
                ctx.hard_hash(q0, W0, 1)
                ctx.score_keys(codes0, length, 1, scores)
            else:
                ctx.score(q0, codes0, W0, tau, length, 1, scores)
            ctx.topk_select(scores, length, k_t, 1, idx, nsel)
            stream.synchronize()
            G = Hq // Hkv
            logits = torch.einsum("hgd,hnd->hgn", q0[0].float().view(Hkv, G, d), K0[0, :, :cur_len].float())
            mass = torch.softmax(logits, dim=-1)
            sel = idx[0].long()                                          # [Hkv, k]
            got_mass = torch.gather(mass, 2, sel[:, None, :].expand(-1, G, -1)).sum(-1)   # [Hkv, G]
            exact = torch.topk(logits.mean(1), k, dim=-1).indices        # [Hkv, k]
            hits = sum(len(set(sel[h].tolist()) & set(exact[h].tolist())) for h in range(Hkv))
            return {"softmax_mass_kept": float(got_mass.mean()), "precision_vs_exact_topk": hits / (Hkv * k)}
        quality = {"soft": selection_quality(False), "hard": selection_quality(True)}

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

    # ---------------- roofline of the dominant kernel (scoring) -------------------------
    # algorithmic bytes per launch: every bucket id read once + one fp32 score written per key
    score_bytes = Hkv * cur_len * (id_bytes + 4)
    score_gbs = score_bytes / (stage_us["score"] * 1e-6) / 1e9
    chain_bytes = Hkv * (cur_len * (id_bytes + 8) + k * (4 * d + 8))
    chain_us = stage_us["fused_decode_step"]
    # HBM bytes per launch from rocprofv3 FETCH_SIZE / WRITE_SIZE, scaled by a plain copy of
    # known size (profiles/score_kernel_128k.md); not measured for other workloads
    traffic = MEASURED_SCORE_TRAFFIC.get((args.workload, NL)) if (L, P) == (64, 8) else None

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
        "keys_scored_per_s": Hkv * cur_len / (stage_us["score"] * 1e-6),
        "layer_step_us": ms_per_step * 1e3 / NL,
        "stage_us_per_layer": stage_us,
        "chain": {"fused_step_us": chain_us, "algorithmic_bytes": chain_bytes,
                  "gbs": chain_bytes / (chain_us * 1e-6) / 1e9,
                  "frac_of_hbm_peak": chain_bytes / (chain_us * 1e-6) / 1e9 / HBM_PEAK_GBS},
        "roofline": {"kernel": "score_kernel" if P <= 8 else "score_split_kernel", "bound": "hbm", "achieved": score_gbs,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": score_gbs / HBM_PEAK_GBS,
                     "traffic": traffic, "algorithmic_bytes": score_bytes,
                     "avg_launch_us": stage_us["score"]},
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

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(layers[0], idx.shape[-1], n, Hq, Hkv, d, L, P, tau, NL,
                                              args.cpu_seconds)
    print(json.dumps(result))


def cpu_baseline(layer0, k, n, Hq, Hkv, d, L, P, tau, NL, budget_s):
    """The CPU oracle, as it stands, on one layer's share of a decode step (all 8 KV heads of
    layer 0: hash the appended key, soft-hash 4 queries per head, score n keys, full-sort
    top-k, attention over the k rows), repeated for about `budget_s` seconds."""
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    import numpy as np
    import harness as hz
    import oracle

    K, V, q, W, codes = layer0
    Kh = K[0, :, :n + 1].float().cpu().numpy()
    Vh = V[0, :, :n + 1].float().cpu().numpy()
    qh = q[0].float().cpu().numpy()
    Wh = W.float().cpu().numpy()
    rows = hz.rows_from_device(codes.view(1, Hkv, -1, hz.lpad_of(L) * (1 if P <= 8 else 2)) if not hz.packed(P)
                               else codes.view(1, Hkv, -1, 20 * hz.lpad_of(L)), L, P)
    nat = hz.codes_to_natural(rows[0, :, :n + 1], L, P=P).astype(np.uint16)
    G = Hq // Hkv

    def layer_step():
        for h in range(Hkv):
            new_code, _ = oracle.hash_keys(Kh[h, n:n + 1], Wh[h], L, P)
            c = nat[h].copy()
            c[n] = new_code[0]
            p = np.stack([oracle.soft_probs(qh[h * G + g], Wh[h], L, P, tau) for g in range(G)])
            s = oracle.score(c, p, P)
            sel, cnt = oracle.topk(s, k)
            for g in range(G):
                oracle.sparse_decode(qh[h * G + g], Kh[h], Vh[h], sel[:cnt], 1.0)

    layer_step()
    reps, t0 = 0, time.perf_counter()
    while True:
        layer_step()
        reps += 1
        el = time.perf_counter() - t0
        if el >= budget_s or reps >= 50:
            break
    per_layer = el / reps
    return {"value": 1.0 / (per_layer * NL), "unit": "steps/s", "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": f"{reps} layer-steps of layer 0 (8 KV heads, ctx {n}) in {el:.1f} s; "
                      f"a decode step is {NL} layer-steps, so value = 1/({NL} x {per_layer:.3f} s)"}


if __name__ == "__main__":
    main()
