"""socket_sparse_decode_noalloc (no context, split-K partial results in a fixed device array)
against socket_sparse_decode on the same inputs: same kernels, so the outputs must agree bit
for bit, and both must agree with the oracle's Eq. 2 to the attention tolerance.  Two calls in
a row share the array; the second is smaller (fewer sequences, fewer selected tokens, fewer
splits), so anything the first left behind would show."""
import numpy as np
import pytest
import torch

import harness as hz
import oracle
from paper_2602_06283_amd import binding as sk
from paper_2602_06283_amd import workloads as wl

pytestmark = pytest.mark.gpu


def one_case(seed, B, Hq, Hkv, d, n, k, lens, kv_dtype, out_dtype, atol):
    layer = wl.make_layer(seed, B=B, Hq=Hq, Hkv=Hkv, d=d, n=n, L=16, P=4, k=k, kv_dtype=kv_dtype, seq_len=lens)
    rng = np.random.default_rng(seed)
    max_k = int(layer.k.max())
    idx = np.full((B, Hkv, max_k), -1, dtype=np.int32)
    nsel = np.zeros((B, Hkv), dtype=np.int32)
    for b in range(B):
        for h in range(Hkv):
            cnt = min(int(layer.k[b]), int(layer.seq_len[b]))
            idx[b, h, :cnt] = np.sort(rng.choice(int(layer.seq_len[b]), size=cnt, replace=False))
            nsel[b, h] = cnt
    Kd, Vd, qd = (hz.dev(x, layer.kv_dtype) for x in (layer.K, layer.V, layer.q))
    idx_d, nsel_d = hz.i32(idx), hz.i32(nsel)
    ctx = hz.make_ctx(layer)
    want = torch.zeros((B, Hq, d), dtype=out_dtype, device="cuda")
    ctx.sparse_decode(qd, Kd, Vd, idx_d, nsel_d, B, 1.0, want)
    got = torch.full((B, Hq, d), 7.0, dtype=out_dtype, device="cuda")
    sk.sparse_decode_noalloc(ctx.params, qd, Kd, Vd, idx_d, nsel_d, B, 1.0, got)
    torch.cuda.synchronize()
    assert torch.equal(got, want)
    got_h = got.float().cpu().numpy()
    G = Hq // Hkv
    for b in range(B):
        for h in range(Hkv):
            y = hz.oracle_attention(layer, b, h, idx[b, h])
            assert np.abs(got_h[b, h * G:(h + 1) * G] - y).max() <= atol
    ctx.close()


def test_noalloc_matches_sparse_decode_twice_second_call_smaller():
    assert torch.cuda.is_available()
    one_case(201, B=3, Hq=8, Hkv=2, d=128, n=4096, k=[1500, 700, 64], lens=[4096, 3000, 100],
             kv_dtype=wl.BF16, out_dtype=torch.float32, atol=1e-4)
    one_case(202, B=1, Hq=2, Hkv=1, d=64, n=512, k=[40], lens=[300], kv_dtype=wl.F32,
             out_dtype=torch.float32, atol=1e-4)
    one_case(203, B=2, Hq=4, Hkv=4, d=128, n=2048, k=[300, 1], lens=[2048, 7], kv_dtype=wl.BF16,
             out_dtype=torch.bfloat16, atol=2e-2)


def test_noalloc_rejects_what_the_fixed_array_cannot_hold():
    assert torch.cuda.is_available()
    # 16 sequences x 32 query heads x 64 splits x 130 floats = 17 MB > 4 MiB
    p = sk.make_params(128, 32, 8, 16, 4, sk.BF16, 16, 8192, 4096)
    t = torch.zeros(16, dtype=torch.float32, device="cuda")
    with pytest.raises(sk.SocketError) as e:
        sk.sparse_decode_noalloc(p, t, t, t, t, t, 16, 1.0, t)
    assert e.value.code == sk.ELIMIT
