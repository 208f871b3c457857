"""Seeded synthetic inputs for the SOCKET decode path.

This module only draws random tensors and lays them out; it holds none of the
method's arithmetic (no hashing, scoring, selection or attention) and imports
neither the GPU binding nor the CPU oracle.  Both consume what it returns.

The paper measures on attention layers of Llama-3.1-8B fed long-context prompts;
those activations are not available, so tensors of the same shapes with Gaussian
entries, outlier channels and a few keys planted close to the query stand in for
them.  All floating-point tensors are returned as float32 numpy arrays whose
values are exactly representable in the stated storage type (bf16 values are
rounded once, here, with round-to-nearest-even), so a consumer may narrow them
to that type without changing any value.
"""
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

BF16 = "bf16"
F32 = "f32"


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result stays float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = (bits + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """The 16 storage bits of bf16-representable float32 values (uint16 array)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    return round_to_bf16(x) if dtype == BF16 else np.ascontiguousarray(x, dtype=np.float32)


def make_projection(seed: int, Hkv: int, d: int, L: int, P: int, dtype: str) -> np.ndarray:
    """Gaussian hyperplanes, one set per KV head: [Hkv, d, L*P], N(0,1), stored in `dtype`."""
    rng = np.random.default_rng([seed, 7])
    W = rng.standard_normal((Hkv, d, L * P), dtype=np.float32)
    return _store(W, dtype)


@dataclass
class Layer:
    """One decode-attention layer's inputs in logical (contiguous) layout."""
    B: int
    Hq: int
    Hkv: int
    d: int
    n: int                    # tokens allocated per sequence (max over the batch)
    L: int
    P: int
    k: np.ndarray             # [B] int32, tokens to select per sequence
    kv_dtype: str
    seq_len: np.ndarray       # [B] int32
    K: np.ndarray             # [B, Hkv, n, d] float32 (values exact in kv_dtype)
    V: np.ndarray             # [B, Hkv, n, d]
    q: np.ndarray             # [B, Hq, d]
    W: np.ndarray             # [Hkv, d, L*P]
    planted: list = field(default_factory=list)   # planted[b][h] = sorted positions
    tau: float = 0.5
    scale: float = 1.0

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv


def make_layer(seed: int, B: int, Hq: int, Hkv: int, d: int, n: int, L: int, P: int, k,
               kv_dtype: str = BF16, seq_len=None, channel_sigma: float = 0.5,
               planted_frac: float = 0.01, planted_count: Optional[int] = None,
               plant_coef: float = 0.7, plant_noise: Optional[float] = None,
               tau: float = 0.5) -> Layer:
    """Draw one layer.

    Keys are N(0,1) times a per-channel scale drawn LogNormal(0, channel_sigma) per
    KV head (channel_sigma = 0 gives plain N(0,1)); values and queries are N(0,1).
    A fraction `planted_frac` (or exactly `planted_count`) of each head's valid
    positions is overwritten with  plant_coef * q_g + plant_noise * N(0,1), where g
    is drawn uniformly from the query heads sharing that KV head.  plant_noise
    defaults to sqrt(1 - plant_coef^2).
    """
    assert Hq % Hkv == 0
    G = Hq // Hkv
    rng = np.random.default_rng([seed, 1])
    if seq_len is None:
        seq_len = np.full(B, n, dtype=np.int32)
    seq_len = np.asarray(seq_len, dtype=np.int32)
    assert seq_len.shape == (B,) and int(seq_len.max(initial=0)) <= n
    if plant_noise is None:
        plant_noise = float(np.sqrt(max(0.0, 1.0 - plant_coef * plant_coef)))

    q = rng.standard_normal((B, Hq, d), dtype=np.float32)
    q = _store(q, kv_dtype)
    K = rng.standard_normal((B, Hkv, n, d), dtype=np.float32)
    if channel_sigma > 0:
        s = np.exp(channel_sigma * rng.standard_normal((Hkv, d))).astype(np.float32)
        K *= s[None, :, None, :]
    V = rng.standard_normal((B, Hkv, n, d), dtype=np.float32)

    planted = []
    for b in range(B):
        per_head = []
        valid = int(seq_len[b])
        cnt = planted_count if planted_count is not None else int(round(planted_frac * valid))
        cnt = min(cnt, valid)
        for h in range(Hkv):
            if cnt == 0:
                per_head.append(np.zeros(0, dtype=np.int64))
                continue
            pos = np.sort(rng.choice(valid, size=cnt, replace=False))
            g = rng.integers(0, G, size=cnt)
            noise = rng.standard_normal((cnt, d), dtype=np.float32)
            K[b, h, pos, :] = plant_coef * q[b, h * G + g, :] + plant_noise * noise
            per_head.append(pos)
        planted.append(per_head)

    K = _store(K, kv_dtype)
    V = _store(V, kv_dtype)
    W = make_projection(seed, Hkv, d, L, P, kv_dtype)
    k = np.broadcast_to(np.asarray(k, dtype=np.int32), (B,)).copy()
    return Layer(B=B, Hq=Hq, Hkv=Hkv, d=d, n=n, L=L, P=P, k=k, kv_dtype=kv_dtype,
                 seq_len=seq_len, K=K, V=V, q=q, W=W, planted=planted, tau=tau)


def draw_step(seed: int, step: int, layer: Layer):
    """New (k, v, q) rows for decode step `step`: k_new,v_new [B,Hkv,d], q [B,Hq,d]."""
    rng = np.random.default_rng([seed, 2, step])
    k_new = _store(rng.standard_normal((layer.B, layer.Hkv, layer.d), dtype=np.float32), layer.kv_dtype)
    v_new = _store(rng.standard_normal((layer.B, layer.Hkv, layer.d), dtype=np.float32), layer.kv_dtype)
    q = _store(rng.standard_normal((layer.B, layer.Hq, layer.d), dtype=np.float32), layer.kv_dtype)
    return k_new, v_new, q


# ---- the five benchmark configurations -------------------------------------------------

def config_tiny(seed: int = 1000) -> Layer:
    """Single head, d=128, n=4096, fp32, L=32, P=8, k=128; 32 keys planted as 0.8 q + 0.6 N(0,1)."""
    return make_layer(seed, B=1, Hq=1, Hkv=1, d=128, n=4096, L=32, P=8, k=128, kv_dtype=F32,
                      channel_sigma=0.0, planted_count=32, plant_coef=0.8, plant_noise=0.6)


def config_llama(n: int, k: int, seed: int, L: int = 64, P: int = 8, B: int = 1) -> Layer:
    """Llama-3-8B-shaped layer: 32 query heads, 8 KV heads, d=128, bf16 KV, 1 % planted keys."""
    return make_layer(seed, B=B, Hq=32, Hkv=8, d=128, n=n, L=L, P=P, k=k, kv_dtype=BF16)


def config_32k(seed: int = 1001) -> Layer:
    return config_llama(32768, 1024, seed)


def config_128k(seed: int = 1002) -> Layer:
    return config_llama(131072, 2048, seed)


def config_batched_lengths(seed: int = 1003, B: int = 16, lo: int = 8192, hi: int = 32768):
    """Per-sequence lengths ~ U[lo, hi] and k = max(256, ceil(2 % of length))."""
    rng = np.random.default_rng([seed, 3])
    lens = rng.integers(lo, hi + 1, size=B).astype(np.int32)
    k = np.maximum(256, np.ceil(0.02 * lens)).astype(np.int32)
    return lens, k


# ---- paged layout -----------------------------------------------------------------------

def make_block_table(seed: int, seq_capacity: np.ndarray, page: int):
    """Random block table: block_table [B, max_blocks] int32 (unused = -1), num_blocks.

    seq_capacity[b] = tokens sequence b must be able to hold (current length plus
    the rows that later decode steps append).
    """
    rng = np.random.default_rng([seed, 4])
    blocks_per_seq = [(int(c) + page - 1) // page for c in seq_capacity]
    total = int(sum(blocks_per_seq))
    perm = rng.permutation(total).astype(np.int32)
    table = np.full((len(blocks_per_seq), max(blocks_per_seq)), -1, dtype=np.int32)
    at = 0
    for b, nb in enumerate(blocks_per_seq):
        table[b, :nb] = perm[at:at + nb]
        at += nb
    return table, total


def to_paged(X: np.ndarray, seq_len: np.ndarray, block_table: np.ndarray, num_blocks: int,
             page: int) -> np.ndarray:
    """Scatter logical [B, Hkv, n, d] rows into a pool [num_blocks, Hkv, page, d]."""
    B, Hkv, n, d = X.shape
    pool = np.zeros((num_blocks, Hkv, page, d), dtype=X.dtype)
    for b in range(B):
        ln = int(seq_len[b])
        nb = (ln + page - 1) // page
        for i in range(nb):
            lo = i * page
            hi = min(ln, lo + page)
            pool[block_table[b, i], :, : hi - lo, :] = X[b, :, lo:hi, :]
    return pool


# ---- device-side generator for the benchmark's many layers ------------------------------

def device_layer(seed: int, Hq: int, Hkv: int, d: int, n: int, n_alloc: int, L: int, P: int,
                 channel_sigma: float = 0.5, planted_frac: float = 0.01, plant_coef: float = 0.7,
                 device: str = "cuda"):
    """Same recipe as make_layer (B = 1, bf16), drawn on the GPU with torch's generator so that
    tens of layers of a 128K-token cache can be filled in seconds.  Rows [n, n_alloc) are
    filled too: they are the keys/values that later decode steps "append".
    Returns K, V [1, Hkv, n_alloc, d] bf16, q [1, Hq, d] bf16, W [Hkv, d, L*P] bf16."""
    import torch
    G = Hq // Hkv
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    q = torch.randn((1, Hq, d), generator=gen, device=device, dtype=torch.float32)
    scale = torch.exp(channel_sigma * torch.randn((Hkv, 1, d), generator=gen, device=device))
    K = torch.empty((1, Hkv, n_alloc, d), device=device, dtype=torch.bfloat16)
    V = torch.empty((1, Hkv, n_alloc, d), device=device, dtype=torch.bfloat16)
    cnt = int(round(planted_frac * n))
    noise_w = float(np.sqrt(max(0.0, 1.0 - plant_coef * plant_coef)))
    for h in range(Hkv):            # one head at a time keeps the fp32 temporaries small
        k = torch.randn((n_alloc, d), generator=gen, device=device) * scale[h]
        if cnt:
            pos = torch.randperm(n, generator=gen, device=device)[:cnt]
            g = torch.randint(0, G, (cnt,), generator=gen, device=device)
            k[pos] = plant_coef * q[0, h * G + g] + noise_w * torch.randn((cnt, d), generator=gen, device=device)
        K[0, h] = k.to(torch.bfloat16)
        V[0, h] = torch.randn((n_alloc, d), generator=gen, device=device).to(torch.bfloat16)
    W = torch.randn((Hkv, d, L * P), generator=gen, device=device).to(torch.bfloat16)
    return K, V, q.to(torch.bfloat16), W


def device_batch(seed: int, B: int, Hq: int, Hkv: int, d: int, n: int, n_alloc: int,
                 channel_sigma: float = 0.5, planted_frac: float = 0.01, plant_coef: float = 0.7,
                 device: str = "cuda"):
    """make_layer's recipe for B sequences of n tokens in contiguous caches, drawn on the GPU:
    K, V [B, Hkv, n_alloc, d] bf16 (rows [n, n_alloc) filled too: the rows decode steps append),
    q [B, Hq, d] bf16.  No projection: the caller draws the hyperplanes it wants."""
    import torch
    G = Hq // Hkv
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    q = torch.randn((B, Hq, d), generator=gen, device=device, dtype=torch.float32)
    scale = torch.exp(channel_sigma * torch.randn((Hkv, 1, d), generator=gen, device=device))
    K = torch.empty((B, Hkv, n_alloc, d), device=device, dtype=torch.bfloat16)
    V = torch.empty((B, Hkv, n_alloc, d), device=device, dtype=torch.bfloat16)
    cnt = int(round(planted_frac * n))
    noise_w = float(np.sqrt(max(0.0, 1.0 - plant_coef * plant_coef)))
    for b in range(B):
        for h in range(Hkv):
            k = torch.randn((n_alloc, d), generator=gen, device=device) * scale[h]
            if cnt:
                pos = torch.randperm(n, generator=gen, device=device)[:cnt]
                g = torch.randint(0, G, (cnt,), generator=gen, device=device)
                k[pos] = plant_coef * q[b, h * G + g] + noise_w * torch.randn((cnt, d), generator=gen, device=device)
            K[b, h] = k.to(torch.bfloat16)
            V[b, h] = torch.randn((n_alloc, d), generator=gen, device=device).to(torch.bfloat16)
    return K, V, q.to(torch.bfloat16)


def device_paged_layer(seed: int, B: int, Hq: int, Hkv: int, d: int, lens, cap: int, page: int,
                       block_table: np.ndarray, num_blocks: int, L: int, P: int, n_steps: int,
                       channel_sigma: float = 0.5, planted_frac: float = 0.01, plant_coef: float = 0.7,
                       device: str = "cuda"):
    """make_layer's recipe for B sequences of lens[b] tokens, written into paged pools through
    `block_table`: K, V [num_blocks, Hkv, page, d] bf16 (every sequence's rows up to `cap` are
    filled: those beyond lens[b] are what decode steps append), queries for n_steps decode
    steps [n_steps, B, Hq, d] bf16 (the planted keys lean on step 0's queries), W [Hkv, d, L*P]."""
    import torch
    G = Hq // Hkv
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    qs = torch.randn((n_steps, B, Hq, d), generator=gen, device=device, dtype=torch.float32)
    scale = torch.exp(channel_sigma * torch.randn((Hkv, 1, d), generator=gen, device=device))
    K = torch.zeros((num_blocks, Hkv, page, d), device=device, dtype=torch.bfloat16)
    V = torch.zeros((num_blocks, Hkv, page, d), device=device, dtype=torch.bfloat16)
    noise_w = float(np.sqrt(max(0.0, 1.0 - plant_coef * plant_coef)))
    nb = cap // page
    for b in range(B):
        blocks = torch.from_numpy(np.ascontiguousarray(block_table[b, :nb]).astype(np.int64)).to(device)
        n = int(lens[b])
        cnt = int(round(planted_frac * n))
        for h in range(Hkv):
            k = torch.randn((cap, d), generator=gen, device=device) * scale[h]
            if cnt:
                pos = torch.randperm(n, generator=gen, device=device)[:cnt]
                g = torch.randint(0, G, (cnt,), generator=gen, device=device)
                k[pos] = plant_coef * qs[0, b, h * G + g] + noise_w * torch.randn((cnt, d), generator=gen, device=device)
            K[blocks, h] = k.to(torch.bfloat16).view(nb, page, d)
            V[blocks, h] = torch.randn((cap, d), generator=gen, device=device).to(torch.bfloat16).view(nb, page, d)
    W = torch.randn((Hkv, d, L * P), generator=gen, device=device).to(torch.bfloat16)
    return K, V, qs.to(torch.bfloat16), W
