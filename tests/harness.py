"""Glue shared by the GPU parity tests, the smoke check and the benchmark: moves the seeded
inputs to the device, re-indexes bucket-id rows between the library's rotated layout and
plain [token, table] order, and runs the CPU oracle per (sequence, KV head).

Nothing here computes any part of the method; it only reshapes, copies and calls.
"""
import numpy as np
import torch

import oracle
from paper_2602_06283_amd import binding as sk
from paper_2602_06283_amd import workloads as wl


def dev(x: np.ndarray, kv_dtype: str) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    return t.to(torch.bfloat16) if kv_dtype == wl.BF16 else t.float()


def i32(x) -> torch.Tensor:
    return torch.tensor(np.asarray(x, dtype=np.int32), dtype=torch.int32, device="cuda")


def pack_factor(L: int, P: int) -> int:
    """Ids of 1, 2 or 4 bits share bytes, 8/P of them, when L is a multiple of that and the bytes
    per token come to 32..128 (see socket.h)."""
    f = 8 // P if P in (1, 2, 4) else 1
    return f if L % f == 0 and 32 <= L // f <= 128 else 1


def lpad_of(L: int, P: int = 8) -> int:
    """Elements of a token's code row."""
    L //= pack_factor(L, P)
    if L <= 16:
        return 16
    if L <= 32:
        return 32
    if L <= 64:
        return 64
    return (L + 63) // 64 * 64


def packed(P: int) -> bool:
    """P = 9 and 10 keep their ids in the packed 10-bit layout (see socket.h)."""
    return P in (9, 10)


def positions(L: int, n: int, P: int = 8) -> np.ndarray:
    """pos[t, l] = where table l's id sits in token t's Lpad-long code row (see socket.h); ids
    that share bytes: the position of the byte that holds it."""
    pf = pack_factor(L, P)
    if pf > 1:
        return np.repeat(positions(L // pf, n, 8), pf, axis=1)
    Lpad = lpad_of(L)
    l = np.arange(L)[None, :]
    t = np.arange(n)[:, None]
    if packed(P):                       # groups of GT tables, S = GT/16 position groups each
        GT = min(Lpad, 32)
        S = GT // 16
        c, lp = l // GT, l % GT
        return GT * c + (lp % S) * 16 + ((lp // S - t) % 16)
    S = 4 if Lpad >= 64 else Lpad // 16
    c = l // 64 if Lpad >= 64 else np.zeros_like(l)
    lp = l - 64 * c
    return 64 * c + (lp % S) * 16 + ((lp // S - t) % 16)


def codes_to_natural(codes: np.ndarray, L: int, t0: int = 0, P: int = 8) -> np.ndarray:
    """[..., n, Lpad] code rows in the library's order -> [..., n, L]; row i is token t0 + i."""
    n = codes.shape[-2]
    pos = positions(L, t0 + n, P)[t0:]
    nat = np.take_along_axis(codes, np.broadcast_to(pos, codes.shape[:-1] + (L,)), axis=-1)
    pf = pack_factor(L, P)
    if pf > 1:                          # field l % pf of the shared byte
        nat = (nat >> (P * (np.arange(L) % pf)).astype(nat.dtype)) & nat.dtype.type((1 << P) - 1)
    return nat


def codes_from_natural(nat: np.ndarray, L: int, dtype, P: int = 8) -> np.ndarray:
    """[..., n, L] -> [..., n, Lpad] code rows in the library's order (padding positions 0)."""
    pf = pack_factor(L, P)
    if pf > 1:                          # pf ids to a byte, then the byte as an 8-bit id of table l // pf
        fields = nat.reshape(nat.shape[:-1] + (L // pf, pf)).astype(np.uint32)
        byte = (fields << (P * np.arange(pf)).astype(np.uint32)).sum(axis=-1)
        return codes_from_natural(byte, L // pf, dtype, 8)
    n = nat.shape[-2]
    out = np.zeros(nat.shape[:-1] + (lpad_of(L),), dtype=dtype)
    pos = positions(L, n, P)
    np.put_along_axis(out, np.broadcast_to(pos, nat.shape), nat.astype(dtype), axis=-1)
    return out


def code_dtype(P: int):
    return np.uint8 if P <= 8 else np.uint16


def torch_code_dtype(P: int):
    return torch.uint8 if P <= 8 or packed(P) else torch.int16


def fill_id(P: int) -> int:
    """What an id reads as where the buffer still holds the 0x55 fill bytes."""
    return 0x55 if P <= 8 else (0x155 if packed(P) else 0x5555)


def new_codes(lead, n: int, L: int, P: int, fill: int = 0) -> torch.Tensor:
    """Device bucket-id buffer for `lead` (sequences or blocks, KV heads) x n tokens, every
    byte = fill.  Unpacked: [*lead, n, Lpad] uint8 / int16; packed: [*lead, n/16, 20*Lpad] bytes."""
    Lpad = lpad_of(L, P)
    if packed(P):
        assert n % 16 == 0
        return torch.full(tuple(lead) + (n // 16, 20 * Lpad), fill, dtype=torch.uint8, device="cuda")
    if P <= 8:
        return torch.full(tuple(lead) + (n, Lpad), fill, dtype=torch.uint8, device="cuda")
    return torch.full(tuple(lead) + (n, Lpad), fill | (fill << 8), dtype=torch.int32, device="cuda").to(torch.int16)


def rows_from_device(raw, L: int, P: int) -> np.ndarray:
    """Bucket-id buffer in the library's storage form (tensor or array, shaped as new_codes
    makes it) -> code rows [..., n, Lpad]."""
    if isinstance(raw, torch.Tensor):
        raw = raw.cpu().numpy()
    if not packed(P):
        return raw.view(code_dtype(P))
    Lpad = lpad_of(L)
    GT = min(Lpad, 32)
    S = GT // 16
    lead, tiles = raw.shape[:-2], raw.shape[-2]
    rows = np.zeros(lead + (tiles, 16, Lpad), dtype=np.uint16)
    weights = (1 << np.arange(10)).astype(np.uint16)
    for g in range(Lpad // GT):
        blk = raw[..., g * 20 * GT:(g + 1) * 20 * GT]
        main = blk[..., :16 * GT].reshape(lead + (tiles, 16, S, 16))
        tail = blk[..., 16 * GT:].reshape(lead + (tiles, 16, S, 4))
        string = np.concatenate([main, tail], axis=-1)                  # 20 bytes = 16 ids of 10 bits
        bits = np.unpackbits(string, axis=-1, bitorder="little").reshape(lead + (tiles, 16, S, 16, 10))
        ids = (bits.astype(np.uint16) * weights).sum(axis=-1).astype(np.uint16)
        rows[..., g * GT:(g + 1) * GT] = ids.reshape(lead + (tiles, 16, GT))
    return rows.reshape(lead + (tiles * 16, Lpad))


def rows_to_device(rows: np.ndarray, L: int, P: int) -> torch.Tensor:
    return torch.from_numpy(rows_to_storage(rows, L, P)).cuda()


def rows_to_storage(rows: np.ndarray, L: int, P: int) -> np.ndarray:
    """Code rows [..., n, Lpad] -> the library's storage form (host array; int16 for two-byte ids)."""
    if not packed(P):
        r = np.ascontiguousarray(rows.astype(code_dtype(P)))
        return r.view(np.uint8 if P <= 8 else np.int16)
    Lpad = lpad_of(L)
    GT = min(Lpad, 32)
    S = GT // 16
    lead, n = rows.shape[:-2], rows.shape[-2]
    assert n % 16 == 0 and rows.shape[-1] == Lpad
    r = rows.reshape(lead + (n // 16, 16, Lpad)).astype(np.uint16)
    raw = np.zeros(lead + (n // 16, 20 * Lpad), dtype=np.uint8)
    for g in range(Lpad // GT):
        ids = r[..., g * GT:(g + 1) * GT].reshape(lead + (n // 16, 16, S, 16))
        bits = ((ids[..., None] >> np.arange(10).astype(np.uint16)) & 1).astype(np.uint8)
        string = np.packbits(bits.reshape(lead + (n // 16, 16, S, 160)), axis=-1, bitorder="little")
        raw[..., g * 20 * GT:g * 20 * GT + 16 * GT] = string[..., :16].reshape(lead + (n // 16, 16 * GT))
        raw[..., g * 20 * GT + 16 * GT:(g + 1) * 20 * GT] = string[..., 16:].reshape(lead + (n // 16, 4 * GT))
    return raw


def make_ctx(layer: wl.Layer, max_k=None, page=0, max_blocks=0, num_blocks=0, max_n=None):
    p = sk.make_params(layer.d, layer.Hq, layer.Hkv, layer.L, layer.P,
                       sk.BF16 if layer.kv_dtype == wl.BF16 else sk.F32, layer.B,
                       max_n if max_n is not None else layer.n,
                       int(max_k if max_k is not None else layer.k.max()), page, max_blocks, num_blocks)
    return sk.Context(p)


# ---- oracle per (sequence, KV head) --------------------------------------------------

def oracle_codes(layer: wl.Layer, b: int, h: int, rows=None):
    K = layer.K[b, h] if rows is None else layer.K[b, h][rows]
    return oracle.hash_keys(K, layer.W[h], layer.L, layer.P)


def oracle_probs(layer: wl.Layer, b: int, h: int, tau=None, q=None):
    tau = layer.tau if tau is None else tau
    q = layer.q if q is None else q
    G = layer.G
    return np.stack([oracle.soft_probs(q[b, h * G + g], layer.W[h], layer.L, layer.P, tau)
                     for g in range(G)])


def oracle_scores(layer: wl.Layer, b: int, h: int, codes_nat, tau=None, vnorm=None, seq_len=None, q=None):
    p = oracle_probs(layer, b, h, tau, q)
    return oracle.score(codes_nat, p, layer.P, vnorm=vnorm,
                        seq_len=int(layer.seq_len[b]) if seq_len is None else seq_len)


def oracle_attention(layer: wl.Layer, b: int, h: int, idx, q=None):
    q = layer.q if q is None else q
    G = layer.G
    return np.stack([oracle.sparse_decode(q[b, h * G + g], layer.K[b, h], layer.V[b, h], idx, layer.scale)
                     for g in range(G)])


def topk_sets_agree(got_idx, want_idx, scores32, margin=1e-6):
    """Index sets must agree except for members whose score is within `margin` of the
    k-th largest score (ties and near-ties).  Returns (ok, n_in_margin_swaps)."""
    got, want = set(int(i) for i in got_idx if i >= 0), set(int(i) for i in want_idx if i >= 0)
    if len(got) != len(want):
        return False, 0
    if got == want:
        return True, 0
    kth = min(float(scores32[i]) for i in want)
    diff = got ^ want
    ok = all(abs(float(scores32[i]) - kth) <= margin for i in diff)
    return ok, len(diff) // 2
