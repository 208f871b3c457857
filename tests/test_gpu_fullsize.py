"""Parity at the benchmark's full sizes, in the launch configuration bench.py times: prefill
hash, then one fused decode step (socket_decode_step, one appended key) on a Llama-3-8B-shaped
layer.  configs[1] (32K context) is checked everywhere; configs[2] (128K) checks the bucket
ids on a sample of rows (the oracle's fp64 hashing of a million keys takes too long for a
test) and everything downstream on all keys."""
import numpy as np
import pytest
import torch

import harness as hz
import oracle
from paper_2602_06283_amd import workloads as wl

pytestmark = pytest.mark.gpu


def run_step(layer, n):
    """layer has n + 16 rows allocated and seq_len = n + 1: prefill-hash n rows, then one
    fused decode step appends row n."""
    B, Hkv, cap = layer.B, layer.Hkv, layer.n
    ctx = hz.make_ctx(layer)
    Kd, Vd, qd, Wd = (hz.dev(x, layer.kv_dtype) for x in (layer.K, layer.V, layer.q, layer.W))
    k = int(layer.k.max())
    codes = torch.zeros((B, Hkv, cap, hz.lpad_of(layer.L)), dtype=torch.uint8, device="cuda")
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
