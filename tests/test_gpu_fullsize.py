"""Parity at the benchmark's full sizes, in the launch configuration bench.py times: prefill
hash, then fused decode steps (socket_decode_step, one appended key per sequence) on
Llama-3-8B-shaped layers.  configs[1] (32K context) is checked everywhere; configs[2] (128K)
checks the bucket ids on a sample of rows (the oracle's fp64 hashing of a million keys takes too
long for a test) and everything downstream on all keys; configs[3] (16 paged sequences, 64
appending steps) and the largest point of configs[4] (L = 128, P = 10, 4 x 65536 keys) check the
ids on a sample of rows plus every appended row, and scores, selection and attention of the last
step on every key of every (sequence, head) resp. of a stated sample of them.  The hard scorer
is checked at the largest setting of the cost comparison, (P, L) = (2, 500) on 32768 keys."""
import numpy as np
import pytest
import torch

import harness as hz
import oracle
from paper_2602_06283_amd import binding as sk
from paper_2602_06283_amd import workloads as wl

pytestmark = pytest.mark.gpu


def run_step(layer, n):
    """layer has n + 16 rows allocated and seq_len = n + 1: prefill-hash n rows, then one
    fused decode step appends row n."""
    B, Hkv, cap = layer.B, layer.Hkv, layer.n
    ctx = hz.make_ctx(layer)
    Kd, Vd, qd, Wd = (hz.dev(x, layer.kv_dtype) for x in (layer.K, layer.V, layer.q, layer.W))
    k = int(layer.k.max())
    codes = torch.zeros((B, Hkv, cap, hz.lpad_of(layer.L, layer.P)), dtype=torch.uint8, device="cuda")
    scores = torch.zeros((B, Hkv, cap), dtype=torch.float32, device="cuda")
    idx = torch.zeros((B, Hkv, k), dtype=torch.int32, device="cuda")
    nsel = torch.zeros((B, Hkv), dtype=torch.int32, device="cuda")
    out = torch.zeros((B, layer.Hq, layer.d), dtype=torch.bfloat16, device="cuda")
    ctx.hash_keys(Kd, Wd, hz.i32([0]), hz.i32([n]), B, n, codes)
    ctx.decode_step(qd, Kd, Vd, codes, Wd, layer.tau, hz.i32([n]), hz.i32(layer.k), B, 1.0, scores, idx,
                    nsel, out)
    torch.cuda.synchronize()
    res = (codes.cpu().numpy(), scores.cpu().numpy(), idx.cpu().numpy(), nsel.cpu().numpy(),
           out.float().cpu().numpy())
    ctx.close()
    return res


def check(layer, codes, scores, idx, nsel, out, hash_rows):
    G, ln = layer.G, int(layer.seq_len[0])
    exempt = checked = 0
    for h in range(layer.Hkv):
        got_codes = hz.codes_to_natural(codes[0, h, :ln], layer.L)
        want, near = oracle.hash_keys(layer.K[0, h][hash_rows], layer.W[h], layer.L, layer.P)
        bad = (got_codes[hash_rows] != want) & ~near
        assert not bad.any(), (h, int(bad.sum()))
        exempt += int(near.sum()); checked += want.size
        want_s = hz.oracle_scores(layer, 0, h, np.pad(got_codes, ((0, layer.n - ln), (0, 0))))
        live = np.isfinite(want_s)
        assert live.sum() == ln and np.isneginf(scores[0, h][~live]).all()
        rel = np.abs(scores[0, h][live] - want_s[live]) / want_s[live]
        assert rel.max() <= 1e-5, rel.max()
        want_idx, cnt = oracle.topk(want_s, int(layer.k[0]))
        assert nsel[0, h] == cnt == int(layer.k[0])
        kth = want_s[want_idx[cnt - 1]]
        ok, _ = hz.topk_sets_agree(idx[0, h], want_idx, want_s, margin=max(1e-6, 2e-5 * abs(kth)))
        assert ok
        assert (np.diff(idx[0, h]) > 0).all()
        want_y = hz.oracle_attention(layer, 0, h, idx[0, h])
        assert np.abs(out[0, h * G:(h + 1) * G] - want_y).max() <= 2e-2
    assert exempt <= 1e-3 * checked


def test_llama_32k_every_row():
    """configs[1]: 32 query heads, 8 KV heads, d = 128, n = 32768, bf16, L = 64, P = 8, k = 1024."""
    assert torch.cuda.is_available()
    n = 32768
    layer = wl.make_layer(1001, B=1, Hq=32, Hkv=8, d=128, n=n + 16, L=64, P=8, k=1024, kv_dtype=wl.BF16,
                          seq_len=[n + 1])
    res = run_step(layer, n)
    check(layer, *res, hash_rows=np.arange(n + 1))


def test_llama_128k_sampled_hash_rows():
    """configs[2]: as above with n = 131072, k = 2048; ids checked on every 16th 64-row tile plus
    the appended row, scores / selection / attention on every key."""
    assert torch.cuda.is_available()
    n = 131072
    layer = wl.make_layer(1002, B=1, Hq=32, Hkv=8, d=128, n=n + 16, L=64, P=8, k=2048, kv_dtype=wl.BF16,
                          seq_len=[n + 1])
    res = run_step(layer, n)
    tiles = np.arange(0, n // 64, 16)
    rows = np.concatenate([(tiles[:, None] * 64 + np.arange(64)[None, :]).ravel(), [n - 1, n]])
    check(layer, *res, hash_rows=rows)



# ------------------------------------------------------------------ configs[3] and configs[4]

def paged_pools(layer, table, nblocks, page):
    full = np.full(layer.B, layer.n, dtype=np.int32)
    return wl.to_paged(layer.K, full, table, nblocks, page), wl.to_paged(layer.V, full, table, nblocks, page)


def logical_rows(raw_rows, table, b, h, n_tok, page):
    """code rows [blocks, Hkv, page, Lpad] -> [n_tok, Lpad] of sequence b, head h"""
    nb = (n_tok + page - 1) // page
    return raw_rows[table[b, :nb], h].reshape(nb * page, -1)[:n_tok]


def test_batched_paged_b16_64_appending_steps():
    """configs[3]: 16 sequences of U[8192, 32768] tokens in 16-token blocks behind a random
    block table, L = 64, P = 8, k = max(256, 2 % of the length); 64 consecutive fused decode
    steps, each appending one key/value row per sequence and using a new query.  Checked
    against the oracle: the bucket ids of 256 sampled prefill rows and of all 64 appended rows
    of every (sequence, head); and for the last step the scores of every key, the selection and
    the attention output of every (sequence, head)."""
    assert torch.cuda.is_available()
    B, Hq, Hkv, d, L, P, page, steps = 16, 32, 8, 128, 64, 8, 16, 64
    lens0, _ = wl.config_batched_lengths(1003, B)
    cap = (int(lens0.max()) + steps + page - 1) // page * page
    kk = np.maximum(256, np.ceil(0.02 * (lens0 + steps))).astype(np.int32)
    layer = wl.make_layer(1003, B=B, Hq=Hq, Hkv=Hkv, d=d, n=cap, L=L, P=P, k=kk, kv_dtype=wl.BF16,
                          seq_len=lens0 + steps)
    table, nblocks = wl.make_block_table(1003, np.full(B, cap), page)
    # the rows that the steps append, and each step's queries
    new = [wl.draw_step(1003, s, layer) for s in range(steps)]
    for s, (k_new, v_new, _) in enumerate(new):
        for b in range(B):
            layer.K[b, :, lens0[b] + s] = k_new[b]
            layer.V[b, :, lens0[b] + s] = v_new[b]
    Kp, Vp = paged_pools(layer, table, nblocks, page)
    p = sk.make_params(d, Hq, Hkv, L, P, sk.BF16, B, cap, int(kk.max()), page, table.shape[1], nblocks)
    ctx = sk.Context(p)
    Kd, Vd, Wd = hz.dev(Kp, wl.BF16), hz.dev(Vp, wl.BF16), hz.dev(layer.W, wl.BF16)
    del Kp, Vp
    bt = hz.i32(table)
    codes = hz.new_codes((nblocks, Hkv), page, L, P, fill=0x55)
    scores = torch.zeros((B, Hkv, cap), dtype=torch.float32, device="cuda")
    idx = torch.zeros((B, Hkv, int(kk.max())), dtype=torch.int32, device="cuda")
    nsel = torch.zeros((B, Hkv), dtype=torch.int32, device="cuda")
    out = torch.zeros((B, Hq, d), dtype=torch.float32, device="cuda")
    ctx.hash_keys(Kd, Wd, hz.i32(np.zeros(B)), hz.i32(lens0), B, int(lens0.max()), codes, block_table=bt)
    k_t = hz.i32(kk)
    for s in range(steps):
        qd = hz.dev(new[s][2], wl.BF16)
        ctx.decode_step(qd, Kd, Vd, codes, Wd, 0.5, hz.i32(lens0 + s), k_t, B, 1.0, scores, idx, nsel, out,
                        block_table=bt)
    torch.cuda.synchronize()
    layer.q = new[-1][2]
    raw = hz.rows_from_device(codes, L, P)
    sc, ix, cnt, y = scores.cpu().numpy(), idx.cpu().numpy(), nsel.cpu().numpy(), out.cpu().numpy()
    G = Hq // Hkv
    rng = np.random.default_rng(7)
    exempt = checked = 0
    for b in range(B):
        ln = int(lens0[b]) + steps
        rows = np.concatenate([np.sort(rng.choice(int(lens0[b]), size=256, replace=False)), np.arange(lens0[b], ln)])
        for h in range(Hkv):
            got = hz.codes_to_natural(logical_rows(raw, table, b, h, ln, page), L)
            want, near = oracle.hash_keys(layer.K[b, h][rows], layer.W[h], L, P)
            assert not ((got[rows] != want) & ~near).any(), (b, h)
            exempt += int(near.sum()); checked += want.size
            want_s = hz.oracle_scores(layer, b, h, np.pad(got, ((0, cap - ln), (0, 0))), seq_len=ln)
            live = np.isfinite(want_s)
            assert live.sum() == ln and np.isneginf(sc[b, h][~live]).all()
            assert (np.abs(sc[b, h][live] - want_s[live]) / want_s[live]).max() <= 1e-5
            want_idx, c = oracle.topk(want_s, int(kk[b]))
            assert cnt[b, h] == c == int(kk[b])
            kth = want_s[want_idx[c - 1]]
            ok, _ = hz.topk_sets_agree(ix[b, h, :c], want_idx, want_s, margin=max(1e-6, 2e-5 * abs(kth)))
            assert ok, (b, h)
            assert (np.diff(ix[b, h, :c]) > 0).all() and (ix[b, h, c:] == -1).all()
            want_y = hz.oracle_attention(layer, b, h, ix[b, h, :c])
            assert np.abs(y[b, h * G:(h + 1) * G] - want_y).max() <= 1e-4
    assert exempt <= 1e-3 * checked
    ctx.close()


def test_sweep_largest_point_l128_p10():
    """configs[4] at its largest point: 4 sequences of 65536 keys, 8 KV heads, L = 128 tables of
    P = 10 planes (packed ids), prefill hash then 8 fused decode steps with k = 1024 (the
    benchmark runs more steps; the path they take is the same).  Ids: 192 sampled prefill rows
    plus every appended row of every (sequence, head).  Scores on every key, selection and
    attention: (sequence, head) = (0, 0), (1, 3), (2, 5), (3, 7)."""
    assert torch.cuda.is_available()
    B, Hq, Hkv, d, L, P, n0, steps, k = 4, 32, 8, 128, 128, 10, 65536, 8, 1024
    cap = n0 + 16
    layer = wl.make_layer(1004, B=B, Hq=Hq, Hkv=Hkv, d=d, n=cap, L=L, P=P, k=k, kv_dtype=wl.BF16,
                          seq_len=np.full(B, n0 + steps))
    new = [wl.draw_step(1004, s, layer) for s in range(steps)]
    for s, (k_new, v_new, _) in enumerate(new):
        layer.K[:, :, n0 + s] = k_new
        layer.V[:, :, n0 + s] = v_new
    ctx = hz.make_ctx(layer)
    Kd, Vd, Wd = (hz.dev(x, wl.BF16) for x in (layer.K, layer.V, layer.W))
    codes = hz.new_codes((B, Hkv), cap, L, P, fill=0x55)
    scores = torch.zeros((B, Hkv, cap), dtype=torch.float32, device="cuda")
    idx = torch.zeros((B, Hkv, k), dtype=torch.int32, device="cuda")
    nsel = torch.zeros((B, Hkv), dtype=torch.int32, device="cuda")
    out = torch.zeros((B, Hq, d), dtype=torch.float32, device="cuda")
    ctx.hash_keys(Kd, Wd, hz.i32(np.zeros(B)), hz.i32(np.full(B, n0)), B, n0, codes)
    for s in range(steps):
        ctx.decode_step(hz.dev(new[s][2], wl.BF16), Kd, Vd, codes, Wd, 0.5, hz.i32(np.full(B, n0 + s)),
                        hz.i32(np.full(B, k)), B, 1.0, scores, idx, nsel, out)
    torch.cuda.synchronize()
    layer.q = new[-1][2]
    ln = n0 + steps
    raw = hz.rows_from_device(codes, L, P)
    sc, ix, cnt, y = scores.cpu().numpy(), idx.cpu().numpy(), nsel.cpu().numpy(), out.cpu().numpy()
    G = Hq // Hkv
    rng = np.random.default_rng(8)
    rows = np.concatenate([np.sort(rng.choice(n0, size=192, replace=False)), np.arange(n0, ln)])
    exempt = checked = 0
    for b in range(B):
        for h in range(Hkv):
            got = hz.codes_to_natural(raw[b, h, :ln], L, P=P)
            want, near = oracle.hash_keys(layer.K[b, h][rows], layer.W[h], L, P)
            assert not ((got[rows] != want) & ~near).any(), (b, h)
            exempt += int(near.sum()); checked += want.size
            if (b, h) not in ((0, 0), (1, 3), (2, 5), (3, 7)):
                continue
            want_s = hz.oracle_scores(layer, b, h, np.pad(got, ((0, cap - ln), (0, 0))), seq_len=ln)
            live = np.isfinite(want_s)
            assert (np.abs(sc[b, h][live] - want_s[live]) / want_s[live]).max() <= 1e-5
            assert np.isneginf(sc[b, h][~live]).all()
            want_idx, c = oracle.topk(want_s, k)
            assert cnt[b, h] == c == k
            kth = want_s[want_idx[c - 1]]
            ok, _ = hz.topk_sets_agree(ix[b, h], want_idx, want_s, margin=max(1e-6, 2e-5 * abs(kth)))
            assert ok, (b, h)
            want_y = hz.oracle_attention(layer, b, h, ix[b, h])
            assert np.abs(y[b, h * G:(h + 1) * G] - want_y).max() <= 1e-4
    assert exempt <= 2e-3 * checked
    ctx.close()


def test_hard_scorer_at_the_cost_comparison_shape():
    """The hard LSH scorer at the largest setting of the cost comparison bench.py prints,
    (P, L) = (2, 500), one sequence of 32768 keys, 8 KV heads of 4 queries: the 2-bit ids go four
    to a byte and a byte's look-up returns the sum of its four tables' terms.  Ids: 256 sampled
    rows of every head against the oracle; collision counts (Eq. 3, hard form) on every key of
    every head whose queries have no projection within 1e-4 of zero, exactly; then the selection
    of k = 1024 keys among the (heavily tied) counts and the attention over it."""
    assert torch.cuda.is_available()
    B, Hq, Hkv, d, L, P, n, k = 1, 32, 8, 128, 500, 2, 32768, 1024
    layer = wl.make_layer(1001, B=B, Hq=Hq, Hkv=Hkv, d=d, n=n, L=L, P=P, k=k, kv_dtype=wl.BF16)
    ctx = hz.make_ctx(layer)
    Kd, Vd, qd, Wd = (hz.dev(x, wl.BF16) for x in (layer.K, layer.V, layer.q, layer.W))
    codes = hz.new_codes((B, Hkv), n, L, P, fill=0x55)
    assert codes.numel() == B * Hkv * n * 128        # 125 bytes of ids per key, padded to two 64-byte chunks
    scores = torch.zeros((B, Hkv, n), dtype=torch.float32, device="cuda")
    idx = torch.zeros((B, Hkv, k), dtype=torch.int32, device="cuda")
    nsel = torch.zeros((B, Hkv), dtype=torch.int32, device="cuda")
    out = torch.zeros((B, Hq, d), dtype=torch.float32, device="cuda")
    ctx.hash_keys(Kd, Wd, hz.i32([0]), hz.i32([n]), B, n, codes)
    ctx.hard_hash(qd, Wd, B)
    ctx.score_keys(codes, hz.i32([n]), B, scores)
    ctx.topk_select(scores, hz.i32([n]), hz.i32([k]), B, idx, nsel)
    ctx.sparse_decode(qd, Kd, Vd, idx, nsel, B, 1.0, out)
    torch.cuda.synchronize()
    raw = hz.rows_from_device(codes, L, P)
    sc, ix, cnt, y = scores.cpu().numpy(), idx.cpu().numpy(), nsel.cpu().numpy(), out.cpu().numpy()[0]
    G = Hq // Hkv
    rows = np.sort(np.random.default_rng(9).choice(n, size=256, replace=False))
    exempt = checked = scored = 0
    for h in range(Hkv):
        got = hz.codes_to_natural(raw[0, h], L, P=P)
        want, near = oracle.hash_keys(layer.K[0, h][rows], layer.W[h], L, P)
        assert not ((got[rows] != want) & ~near).any(), h
        exempt += int(near.sum()); checked += want.size
        want_s = np.zeros(n)
        clean = True
        for g in range(G):
            qc, qnear = oracle.hash_keys(layer.q[0, h * G + g][None], layer.W[h], L, P)
            clean = clean and not qnear.any()
            want_s += oracle.hard_score(got.astype(np.uint16), qc[0])
        if not clean:
            continue
        scored += 1
        want_s = (want_s / G).astype(np.float32)
        assert (sc[0, h] == want_s).all(), h
        want_idx, c = oracle.topk(want_s.astype(np.float64), k)
        assert cnt[0, h] == c == k
        assert (ix[0, h] == np.sort(want_idx)).all(), h      # ties go to the smaller position on both sides
        want_y = hz.oracle_attention(layer, 0, h, ix[0, h])
        assert np.abs(y[h * G:(h + 1) * G] - want_y).max() <= 1e-4
    assert exempt <= 2e-3 * checked and scored >= 1
    ctx.close()
