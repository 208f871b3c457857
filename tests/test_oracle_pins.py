"""Pins for the CPU oracle: every function is checked against something other than
itself -- a hand-derived fixture, a closed form, a limit, brute force in exact
arithmetic, or a library routine for the special case it reduces to.

Each pin is chosen so a plausible slip (dropped term, wrong sign, wrong bit
order, transposed operand, missing normalisation) breaks at least one of them.
"""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.special

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rng(seed):
    return np.random.default_rng(seed)


# ------------------------------------------------------------------ Alg. 1: bucket ids

def test_hash_quadrant_fixture():
    """Hand-derived ids (Alg. 1) for axis and diagonal hyperplanes in the plane."""
    W, K, want = [], [], []
    with open(os.path.join(GOLDEN, "hash_quadrants.txt")) as f:
        for line in f:
            t = line.split()
            if not t or t[0].startswith("#"):
                continue
            if t[0] == "W":
                W.append([float(x) for x in t[1:]])
            elif t[0] == "K":
                K.append([float(t[1]), float(t[2])])
                want.append([int(t[3]), int(t[4])])
    codes, _ = oracle.hash_keys(np.array(K), np.array(W), L=2, P=2)
    assert codes.tolist() == want


def test_hash_matches_exact_integer_bruteforce():
    """Small integer K and W: signs decided in exact rational arithmetic (Alg. 1)."""
    rng = _rng(11)
    n, d, L, P = 48, 6, 3, 4
    K = rng.integers(-5, 6, size=(n, d))
    W = rng.integers(-4, 5, size=(d, L * P))
    codes, _ = oracle.hash_keys(K, W, L, P)
    for j in range(n):
        for l in range(L):
            want = 0
            for i in range(P):
                z = sum(Fraction(int(K[j, c])) * int(W[c, l * P + i]) for c in range(d))
                if z >= 0:
                    want |= 1 << i
            assert codes[j, l] == want, (j, l)


def test_hash_is_not_transposed():
    """A non-square, asymmetric W: using W[i][c] for W[c][i] would change the ids."""
    d, L, P = 3, 1, 2
    W = np.array([[1.0, -1.0], [0.0, 2.0], [-3.0, 0.5]])  # [d][L*P]
    K = np.array([[1.0, 1.0, 1.0]])
    # plane 0: 1 + 0 - 3 = -2 -> bit 0 clear; plane 1: -1 + 2 + 0.5 = 1.5 -> bit 1 set
    codes, _ = oracle.hash_keys(K, W, L, P)
    assert codes.tolist() == [[2]]


def test_hash_sign_symmetries():
    """hash(c k) = hash(k) for c > 0; hash(-k) is the bitwise complement (no zero projections)."""
    rng = _rng(12)
    n, d, L, P = 200, 16, 5, 7
    K = rng.standard_normal((n, d)).astype(np.float32)
    W = rng.standard_normal((d, L * P)).astype(np.float32)
    a, nz = oracle.hash_keys(K, W, L, P, zero_margin=1e-9)
    assert not nz.any()
    b, _ = oracle.hash_keys(3.5 * K, W, L, P)
    c, _ = oracle.hash_keys(-K, W, L, P)
    assert (a == b).all()
    assert (c == ((1 << P) - 1 - a)).all()
    assert a.max() < (1 << P)


def test_hash_near_zero_list():
    """|z| < margin marks the table as fragile; exact zero counts as sign +1."""
    W = np.array([[1.0, 1.0], [0.0, 0.0]])            # d=2, L=1, P=2: both planes read x only
    K = np.array([[5e-5, 1.0], [0.5, 1.0], [0.0, 1.0], [-5e-5, 0.0]])
    codes, nz = oracle.hash_keys(K, W, L=1, P=2, zero_margin=1e-4)
    assert nz[:, 0].tolist() == [True, False, True, True]
    assert codes[:, 0].tolist() == [3, 3, 3, 0]


def test_collision_frequency_follows_angular_kernel():
    """Over random hyperplanes Pr[same bucket] = (1 - theta/pi)^P (the SRP collision law)."""
    rng = _rng(13)
    d, P, L = 8, 3, 6000                 # L independent tables = L Monte-Carlo trials
    theta = 1.0
    a = np.zeros(d); a[0] = 1.0
    b = np.zeros(d); b[0] = math.cos(theta); b[1] = math.sin(theta)
    W = rng.standard_normal((d, L * P)).astype(np.float32)
    codes, _ = oracle.hash_keys(np.stack([a, b]), W, L, P)
    freq = float((codes[0] == codes[1]).mean())
    want = (1.0 - theta / math.pi) ** P
    sigma = math.sqrt(want * (1 - want) / L)
    assert abs(freq - want) < 4.5 * sigma


# ------------------------------------------------------------------ Alg. 2: soft bucket probabilities

def _sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x))


def test_probs_sum_to_one_and_peak_at_hard_bucket():
    rng = _rng(21)
    d, L, P = 32, 9, 6
    W = rng.standard_normal((d, L * P)).astype(np.float32)
    for scale in (1.0, 0.05):
        q = (scale * rng.standard_normal(d)).astype(np.float32)
        for tau in (0.1, 0.5, 2.0):
            p = oracle.soft_probs(q, W, L, P, tau)
            assert p.shape == (L, 1 << P)
            np.testing.assert_allclose(p.sum(axis=1), 1.0, rtol=0, atol=1e-13)
            assert (p > 0).all() and (p <= 1).all()
            qcode, _ = oracle.hash_keys(q[None], W, L, P)
            assert (p.argmax(axis=1) == qcode[0]).all()


def test_probs_equal_product_of_sigmoids():
    """A softmax over the corners of {+-1}^P factorises: p(r) = prod_i sigmoid(2 c_{r,i} u_i / tau).
    The right-hand side is computed here in numpy from W and q, independently of the oracle."""
    rng = _rng(22)
    d, L, P, tau = 24, 4, 5, 0.37
    W = rng.standard_normal((d, L * P)).astype(np.float32)
    q = (0.2 * rng.standard_normal(d)).astype(np.float32)
    p = oracle.soft_probs(q, W, L, P, tau)
    z = q.astype(np.float64) @ W.astype(np.float64)            # [L*P]
    u = np.tanh(z).reshape(L, P) / math.sqrt(d)
    for l in range(L):
        for r in range(1 << P):
            want = 1.0
            for i in range(P):
                c = 1.0 if (r >> i) & 1 else -1.0
                want *= _sigmoid(2.0 * c * u[l, i] / tau)
            assert abs(p[l, r] - want) < 1e-13 * max(1.0, want), (l, r)


def test_probs_hand_value_single_plane():
    """d = 4, one table, one plane, W = 1, q = 0.25 each: z = 1, u = tanh(1)/2,
    p(1) = sigmoid(2u/tau), p(0) = 1 - p(1)  (Alg. 2 written out by hand)."""
    W = np.ones((4, 1), dtype=np.float32)
    q = np.full(4, 0.25, dtype=np.float32)
    tau = 0.5
    p = oracle.soft_probs(q, W, 1, 1, tau)
    u = math.tanh(1.0) / 2.0
    want1 = 1.0 / (1.0 + math.exp(-2.0 * u / tau))
    assert abs(p[0, 1] - want1) < 1e-15
    assert abs(p[0, 0] - (1.0 - want1)) < 1e-15
    # 1/sqrt(d) uses the head dimension d (4 here -> 1/2), not P and not L
    assert abs(want1 - 0.8210075) < 1e-6   # tanh(1) = 0.7615942, 2u/tau = 1.5231884


def test_probs_saturated_depend_on_hamming_distance_only():
    """|Wq| large: tanh = +-1, so p(r) = s+^(P-h) s-^h with s+- = sigmoid(+-2/(sqrt(d) tau)),
    h = Hamming distance between r and the query's hard bucket."""
    rng = _rng(23)
    d, L, P, tau = 16, 3, 6, 0.4
    W = rng.standard_normal((d, L * P)).astype(np.float32)
    q = (1000.0 * rng.standard_normal(d)).astype(np.float32)
    p = oracle.soft_probs(q, W, L, P, tau)
    qcode, _ = oracle.hash_keys(q[None], W, L, P)
    sp = _sigmoid(2.0 / (math.sqrt(d) * tau))
    sm = _sigmoid(-2.0 / (math.sqrt(d) * tau))
    for l in range(L):
        for r in range(1 << P):
            h = bin(r ^ int(qcode[0, l])).count("1")
            assert abs(p[l, r] - sp ** (P - h) * sm ** h) < 1e-12


def test_probs_temperature_limits():
    """tau -> 0 puts all mass on the hard bucket; tau -> infinity gives 1/R everywhere."""
    rng = _rng(24)
    d, L, P = 16, 5, 4
    W = rng.standard_normal((d, L * P)).astype(np.float32)
    q = rng.standard_normal(d).astype(np.float32)
    qcode, _ = oracle.hash_keys(q[None], W, L, P)
    cold = oracle.soft_probs(q, W, L, P, 1e-4)
    for l in range(L):
        assert cold[l, qcode[0, l]] > 1 - 1e-9
    hot = oracle.soft_probs(q, W, L, P, 1e6)
    np.testing.assert_allclose(hot, 1.0 / (1 << P), rtol=1e-5)


# ------------------------------------------------------------------ Alg. 5 / Eq. 3: scores

def _setup_scores(seed, n=300, d=16, L=7, P=5, G=1, qscale=1.0):
    rng = _rng(seed)
    W = rng.standard_normal((d, L * P)).astype(np.float32)
    K = rng.standard_normal((n, d)).astype(np.float32)
    qs = (qscale * rng.standard_normal((G, d))).astype(np.float32)
    codes, _ = oracle.hash_keys(K, W, L, P)
    return rng, W, K, qs, codes


def test_score_is_table_lookup_sum_bruteforce():
    """Python-loop restatement of Eq. 3 (soft) on a tiny case, including nu_j and the mask."""
    rng, W, K, qs, codes = _setup_scores(31, n=40, G=2)
    L, P, tau = 7, 5, 0.5
    p = np.stack([oracle.soft_probs(q, W, L, P, tau) for q in qs])
    vn = rng.uniform(0.5, 2.0, size=40).astype(np.float32)
    mask = (rng.uniform(size=40) > 0.2).astype(np.uint8)
    got = oracle.score(codes, p, P, vnorm=vn, mask=mask, seq_len=35)
    for j in range(40):
        if j >= 35 or not mask[j]:
            assert got[j] == -np.inf
            continue
        per_q = [sum(p[g, l, codes[j, l]] for l in range(L)) for g in range(2)]
        want = float(vn[j]) * (sum(per_q) / 2.0)
        assert abs(got[j] - want) < 1e-13
    # nu = 1 when vnorm is absent
    plain = oracle.score(codes, p[0], P)
    want0 = sum(p[0, l, codes[0, l]] for l in range(L))
    assert abs(plain[0] - want0) < 1e-13


def test_score_bounds_and_maximum():
    """Each table contributes a probability, so scores lie in [0, L]; a key in the query's
    own buckets (the query itself, or any positive multiple) gets sum_l max_r p, the maximum."""
    rng, W, K, qs, codes = _setup_scores(32)
    L, P, tau = 7, 5, 0.5
    q = qs[0]
    p = oracle.soft_probs(q, W, L, P, tau)
    K2 = np.vstack([K, q[None], 2.5 * q[None]])
    codes2, _ = oracle.hash_keys(K2, W, L, P)
    s = oracle.score(codes2, p, P)
    assert (s >= 0).all() and (s <= L).all()
    best = p.max(axis=1).sum()
    assert abs(s[-1] - best) < 1e-13 and abs(s[-2] - best) < 1e-13
    assert (s <= best + 1e-13).all()


def test_score_hard_and_flat_limits():
    """tau -> 0: soft score = number of colliding tables (Eq. 3, left); tau -> inf: L/R."""
    rng, W, K, qs, codes = _setup_scores(33, n=500, P=3)
    L, P = 7, 3
    q = qs[0]
    qcode, _ = oracle.hash_keys(q[None], W, L, P)
    hard = oracle.hard_score(codes, qcode[0])
    assert hard.max() >= 2 and hard.min() == 0        # the case is not degenerate
    want = np.array([sum(int(codes[j, l] == qcode[0, l]) for l in range(L)) for j in range(500)])
    assert (hard == want).all()
    cold = oracle.score(codes, oracle.soft_probs(q, W, L, P, 1e-4), P)
    np.testing.assert_allclose(cold, hard, atol=1e-9)
    hot = oracle.score(codes, oracle.soft_probs(q, W, L, P, 1e7), P)
    np.testing.assert_allclose(hot, L / (1 << P), rtol=1e-5)


def test_score_mass_identity():
    """If every bucket of every table holds exactly one key, the scores sum to L
    (sum_j s_j^(l) = sum_r p(r) * #bucket_r with one key per bucket)."""
    rng = _rng(34)
    d, L, P = 12, 6, 4
    R = 1 << P
    W = rng.standard_normal((d, L * P)).astype(np.float32)
    q = rng.standard_normal(d).astype(np.float32)
    codes = np.stack([rng.permutation(R) for _ in range(L)], axis=1).astype(np.uint16)  # [R, L]
    s = oracle.score(codes, oracle.soft_probs(q, W, L, P, 0.3), P)
    assert abs(s.sum() - L) < 1e-12


def test_score_ranks_similar_keys_higher():
    """Sanity of the whole scoring chain: keys close in angle to q outrank random keys on average."""
    rng = _rng(35)
    d, L, P = 64, 48, 8
    W = rng.standard_normal((d, L * P)).astype(np.float32)
    q = rng.standard_normal(d).astype(np.float32)
    K = rng.standard_normal((400, d)).astype(np.float32)
    K[:20] = 0.8 * q + 0.6 * rng.standard_normal((20, d)).astype(np.float32)
    codes, _ = oracle.hash_keys(K, W, L, P)
    s = oracle.score(codes, oracle.soft_probs(q, W, L, P, 0.5), P)
    top, _ = oracle.topk(s, 20)
    assert len(set(top.tolist()) & set(range(20))) >= 17


# ------------------------------------------------------------------ TopK

def test_topk_matches_sort_and_breaks_ties_by_index():
    rng = _rng(41)
    s = rng.standard_normal(257)
    s[10] = s[200] = s[37] = 0.25                 # a three-way tie
    for k in (1, 5, 64, 257):
        idx, cnt = oracle.topk(s, k)
        order = np.lexsort((np.arange(257), -s))   # library sort: score desc, index asc
        assert cnt == k
        assert idx.tolist() == order[:k].tolist()
    idx, _ = oracle.topk(s, 1)
    assert idx[0] == int(np.argmax(s))
    # tie straddling the cut: the smaller indices win
    t = np.zeros(8); t[3] = 1.0
    idx, cnt = oracle.topk(t, 3)
    assert idx.tolist() == [3, 0, 1] and cnt == 3


def test_topk_skips_masked_and_pads():
    s = np.array([0.5, -np.inf, 0.7, -np.inf, 0.1])
    idx, cnt = oracle.topk(s, 4)
    assert cnt == 3 and idx.tolist() == [2, 0, 4, -1]
    idx, cnt = oracle.topk(s, 5)
    assert sorted(idx[:cnt].tolist()) == [0, 2, 4]
    idx, cnt = oracle.topk(np.zeros(0), 3)
    assert cnt == 0 and idx.tolist() == [-1, -1, -1]


def test_topk_bruteforce_tiny():
    """All k-subsets of a tiny array: the selected set has the largest possible score sum."""
    rng = _rng(42)
    s = rng.standard_normal(9)
    idx, _ = oracle.topk(s, 4)
    best = max(itertools.combinations(range(9), 4), key=lambda c: sum(s[list(c)]))
    assert set(idx.tolist()) == set(best)


# ------------------------------------------------------------------ Eq. 1 / Eq. 2: attention

def test_dense_decode_is_textbook_softmax_without_sqrt_d():
    """Eq. 1 against scipy's softmax: logits are k.q with no 1/sqrt(d)."""
    rng = _rng(51)
    n, d = 64, 16
    K = rng.standard_normal((n, d)).astype(np.float32)
    V = rng.standard_normal((n, d)).astype(np.float32)
    q = rng.standard_normal(d).astype(np.float32)
    a = scipy.special.softmax(K.astype(np.float64) @ q.astype(np.float64))
    want = a @ V.astype(np.float64)
    np.testing.assert_allclose(oracle.dense_decode(q, K, V), want, atol=1e-13)
    scaled = scipy.special.softmax((K.astype(np.float64) @ q.astype(np.float64)) / 4.0) @ V.astype(np.float64)
    np.testing.assert_allclose(oracle.dense_decode(q, K, V, scale=0.25), scaled, atol=1e-13)
    assert np.abs(want - scaled).max() > 1e-3      # the factor matters on this input


def test_sparse_decode_reductions():
    """Eq. 2: all indices = Eq. 1; order of indices is irrelevant; one index returns its value
    row; -1 entries are skipped; an empty set gives zeros; a subset equals dense on that subset."""
    rng = _rng(52)
    n, d = 50, 8
    K = (3.0 * rng.standard_normal((n, d))).astype(np.float32)   # logits of order +-25
    V = rng.standard_normal((n, d)).astype(np.float32)
    q = rng.standard_normal(d).astype(np.float32)
    full = oracle.dense_decode(q, K, V)
    np.testing.assert_allclose(oracle.sparse_decode(q, K, V, np.arange(n)), full, atol=1e-13)
    perm = rng.permutation(n)
    np.testing.assert_allclose(oracle.sparse_decode(q, K, V, perm), full, atol=1e-13)
    np.testing.assert_allclose(oracle.sparse_decode(q, K, V, [7]), V[7], atol=1e-15)
    sub = np.array([3, 17, -1, 41, 8, -1])
    keep = sub[sub >= 0]
    a = scipy.special.softmax(K[keep].astype(np.float64) @ q.astype(np.float64))
    np.testing.assert_allclose(oracle.sparse_decode(q, K, V, sub), a @ V[keep].astype(np.float64), atol=1e-13)
    assert (oracle.sparse_decode(q, K, V, [-1, -1]) == 0).all()


def test_attention_shift_invariance_and_large_logits():
    """Adding c q/|q|^2 to every key adds c to every logit and must not change the output;
    logits near +-300 must not overflow."""
    rng = _rng(53)
    n, d = 40, 8
    K = rng.standard_normal((n, d))
    V = rng.standard_normal((n, d)).astype(np.float32)
    q = rng.standard_normal(d)
    base = oracle.dense_decode(q, K, V)
    shifted = K + 300.0 * q / (q @ q)
    out = oracle.dense_decode(q, shifted.astype(np.float32), V)
    assert np.isfinite(out).all()
    np.testing.assert_allclose(out, base, atol=2e-3)   # fp32 storage of the shifted keys limits this


def test_value_norms():
    rng = _rng(54)
    V = rng.standard_normal((33, 12)).astype(np.float32)
    np.testing.assert_allclose(oracle.value_norms(V), np.linalg.norm(V.astype(np.float64), axis=1), rtol=1e-6)


def test_forced_sink_and_window_tokens():
    """Experiments section: sink and local-window tokens are always kept.  Brute force: the
    forced positions are exactly [0, n_sink) and [seq_len - n_window, seq_len); they win the
    TopK step ahead of any finite score, in position order; masked tokens stay masked; tokens
    beyond seq_len are untouched."""
    rng = _rng(55)
    n, seq = 50, 41
    s = rng.standard_normal(n)
    s[3] = -np.inf                      # a masked sink token
    s[seq:] = -np.inf
    out = oracle.force_tokens(s, seq, 4, 6)
    forced = [j for j in range(seq) if (j < 4 or j >= seq - 6) and j != 3]
    assert np.isposinf(out[forced]).all() and np.isneginf(out[3])
    rest = [j for j in range(n) if j not in forced]
    assert (out[rest] == s[rest]).all()
    sel, cnt = oracle.topk(out, 12)
    assert cnt == 12 and sorted(sel[:9].tolist()) == forced and sel[:9].tolist() == forced
    best_free = [j for j in np.argsort(-s[:seq], kind="stable") if j not in forced and j != 3][:3]
    assert sel[9:12].tolist() == best_free
    # windows that overlap or exceed the sequence force every valid token, nothing else
    all_forced = oracle.force_tokens(rng.standard_normal(n), 10, 8, 8)
    assert np.isposinf(all_forced[:10]).all() and np.isfinite(all_forced[10:]).all()
    assert (oracle.force_tokens(s, seq, 0, 0) == s).all()


# ------------------------------------------------------------------ planted mistakes are caught

def test_pins_catch_bit_order_mismatch():
    """If ids used one bit order and corners the other, the query's own bucket would no longer
    be the arg-max.  Emulate the slip by bit-reversing ids and check the pin notices."""
    rng = _rng(61)
    d, L, P = 16, 6, 5
    W = rng.standard_normal((d, L * P)).astype(np.float32)
    q = rng.standard_normal(d).astype(np.float32)
    p = oracle.soft_probs(q, W, L, P, 0.5)
    qcode, _ = oracle.hash_keys(q[None], W, L, P)
    rev = np.array([[int(format(int(c), f"0{P}b")[::-1], 2) for c in qcode[0]]])
    assert (p.argmax(axis=1) == qcode[0]).all()
    assert not (p.argmax(axis=1) == rev[0]).all()


# ------------------------------------------------------------------ ranking metrics (appendix)

def _golden(name):
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "ranking_metrics_worked.txt")
    for line in open(path):
        if line.startswith(name + " "):
            return float(line.split()[1])
    raise KeyError(name)


def test_ranking_metrics_hand_worked_cases():
    """Appendix, metric definitions: values worked by hand (tests/golden/ranking_metrics_worked.txt)."""
    ranked = [3, 2, 3, 0, 1, 2]
    assert abs(oracle.ndcg(ranked, ranked) - _golden("ndcg_same_items")) < 5e-7
    assert abs(oracle.ndcg(ranked, ranked + [3, 2]) - _golden("ndcg_two_missed")) < 5e-7
    assert oracle.precision([1, 2, 3, 4], [2, 4, 6]) == _golden("precision")
    assert abs(oracle.jaccard([1, 2, 3, 4], [2, 4, 6]) - _golden("jaccard")) < 1e-15


def test_ranking_metrics_properties():
    """What the definitions fix for any input: a perfectly ranked list has NDCG 1 and any
    other order of the same items has less; NDCG does not depend on the order of the
    candidate array; identical sets have Jaccard 1 and precision 1, disjoint sets 0; Jaccard
    is symmetric; precision and Jaccard of two k-sets with c common items are c/k and
    c/(2k - c); and both agree with Python's set arithmetic on random sets."""
    rng = _rng(77)
    rel = rng.uniform(0.0, 4.0, size=40)
    order = np.argsort(-rel, kind="stable")
    k = 12
    assert abs(oracle.ndcg(rel[order[:k]], rel) - 1.0) < 1e-15
    swapped = order[:k].copy()
    swapped[[0, k - 1]] = swapped[[k - 1, 0]]
    assert oracle.ndcg(rel[swapped], rel) < 1.0 - 1e-6
    assert oracle.ndcg(rel[swapped], rel) == oracle.ndcg(rel[swapped], rel[rng.permutation(40)])
    worse = order[5:5 + k]                               # misses the five best items
    assert oracle.ndcg(rel[worse], rel) < oracle.ndcg(rel[swapped], rel)
    a = rng.choice(1000, size=50, replace=False)
    assert oracle.jaccard(a, a) == 1.0 and oracle.precision(a, a) == 1.0
    assert oracle.jaccard(a, a + 1000) == 0.0 and oracle.precision(a, a + 1000) == 0.0
    for _ in range(5):
        x = rng.choice(300, size=60, replace=False)
        y = rng.choice(300, size=60, replace=False)
        c = len(set(x.tolist()) & set(y.tolist()))
        assert oracle.precision(x, y) == c / 60
        assert abs(oracle.jaccard(x, y) - c / (120 - c)) < 1e-15
        assert oracle.jaccard(x, y) == oracle.jaccard(y, x)
        z = rng.choice(300, size=25, replace=False)      # sets of different sizes
        assert abs(oracle.jaccard(x, z) - len(set(x.tolist()) & set(z.tolist())) / len(set(x.tolist()) | set(z.tolist()))) < 1e-15
