"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol
the header declares, and its pure-host functions (parameter validation, code layout) behave."""
import os
import re

import numpy as np
import pytest

import harness
from paper_2602_06283_amd import binding as sk

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "socket.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(socket_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert len(names) >= 14
    lib = sk.lib()
    for n in names:
        assert hasattr(lib, n), n
    assert set(sk.EXPORTS) == set(names)


def good():
    return dict(d=128, Hq=32, Hkv=8, L=64, P=8, kv_dtype=sk.BF16, max_batch=1, max_n=4096, max_k=128)


def test_validate_params_accepts_the_benchmark_shapes():
    assert sk.validate_params(sk.make_params(**good())) == sk.OK
    assert sk.validate_params(sk.make_params(128, 1, 1, 32, 8, sk.F32, 1, 4096, 128)) == sk.OK
    for L in (16, 32, 64, 128):
        for P in (4, 8, 10):
            assert sk.validate_params(sk.make_params(128, 32, 8, L, P, sk.BF16, 4, 65536, 1024)) == sk.OK
    for L, P in ((300, 2), (400, 2), (500, 2), (600, 2), (1024, 2), (1024, 1), (256, 4), (258, 4), (7, 4), (1, 1)):
        assert sk.validate_params(sk.make_params(128, 32, 8, L, P, sk.BF16, 1, 32784, 1024)) == sk.OK, (L, P)
    paged = dict(good(), max_batch=16, max_n=32832, max_k=700, page_size=16, max_blocks_per_seq=2052,
                 num_blocks=40000)
    assert sk.validate_params(sk.make_params(**paged)) == sk.OK


@pytest.mark.parametrize("bad", [
    dict(d=100), dict(Hq=30), dict(Hkv=0), dict(L=0), dict(L=2000), dict(P=0), dict(P=17),
    dict(kv_dtype=5), dict(max_batch=0), dict(max_n=100), dict(max_n=8), dict(max_k=0),
    dict(max_k=5000), dict(page_size=24), dict(page_size=16, max_blocks_per_seq=4, num_blocks=9),
    dict(page_size=16, max_blocks_per_seq=0, num_blocks=9),
])
def test_validate_params_rejects(bad):
    assert sk.validate_params(sk.make_params(**dict(good(), **bad))) == sk.EINVAL


def test_unsupported_shapes_are_reported_not_mangled():
    assert sk.validate_params(sk.make_params(**dict(good(), Hq=24))) == sk.EUNSUPPORTED    # G = 3
    assert sk.validate_params(sk.make_params(**dict(good(), P=16))) == sk.EUNSUPPORTED     # table too big for LDS
    assert sk.validate_params(sk.make_params(**dict(good(), Hq=8, P=16, L=16))) == sk.OK   # G = 1 fits


def test_strerror():
    assert sk.strerror(sk.OK) == "ok"
    for c in (sk.EINVAL, sk.EUNSUPPORTED, sk.ENOMEM, sk.EHIP):
        assert sk.strerror(c) and sk.strerror(c) != "ok"


def test_code_layout_matches_documented_formula():
    for L in (1, 7, 16, 24, 32, 60, 64, 100, 128, 300):
        Lpad = sk.codes_per_token(L)
        assert Lpad == harness.lpad_of(L)
        pos = harness.positions(L, 40)
        for t in (0, 1, 5, 15, 16, 17, 39):
            got = [sk.code_position(L, l, t) for l in range(L)]
            assert got == pos[t].tolist()
            assert len(set(got)) == L and max(got) < Lpad      # a permutation into the row
    assert sk.codes_per_token(0) == -1 and sk.codes_per_token(5000) == -1
    assert sk.code_position(64, 64, 0) == -1


def test_layout_round_trip():
    rng = np.random.default_rng(5)
    for L, P in ((24, 8), (64, 8), (128, 4), (60, 10), (16, 9), (100, 10), (40, 12), (300, 2), (16, 4), (66, 4),
                 (7, 4), (256, 1), (600, 2)):
        nat = rng.integers(0, 1 << P, size=(2, 48, L)).astype(harness.code_dtype(P))
        lay = harness.codes_from_natural(nat, L, harness.code_dtype(P), P=P)
        assert lay.shape[-1] == harness.lpad_of(L, P)
        assert (harness.codes_to_natural(lay, L, P=P) == nat).all()
        store = harness.rows_to_storage(lay, L, P)
        assert store.nbytes == 2 * sk.codes_bytes(L, P, 48)
        assert (harness.rows_from_device(store, L, P) == lay).all()


def test_code_location_describes_every_storage_form():
    """socket_code_location against the harness's own packing of random ids: one-byte ids,
    two-byte ids, the packed 10-bit form (whose tiles and groups it has to walk) and ids of 1, 2
    or 4 bits that share bytes (not when L is no multiple of 8/P or the row would not come to 32..128 bytes)."""
    rng = np.random.default_rng(6)
    for L, P in ((64, 8), (24, 5), (60, 10), (64, 9), (16, 10), (128, 10), (40, 12), (300, 2), (128, 4), (16, 4),
                 (66, 4), (7, 4), (256, 1), (600, 2), (2, 2), (64, 4)):
        n = 48
        nat = rng.integers(0, 1 << P, size=(n, L)).astype(harness.code_dtype(P))
        lay = harness.codes_from_natural(nat, L, harness.code_dtype(P), P=P)
        flat = harness.rows_to_storage(lay, L, P).reshape(-1).view(np.uint8)
        assert flat.size == sk.codes_bytes(L, P, n)
        seen = set()
        for t in (0, 1, 15, 16, 17, 31, 47):
            for l in range(L):
                lo, hi, sh = sk.code_location(L, P, l, t)
                got = int(flat[lo])
                if P > 8:
                    got = ((got | int(flat[hi]) << 8) >> sh) & ((1 << P) - 1)
                else:
                    assert hi == -1 and sh == P * (l % harness.pack_factor(L, P))
                    got = (got >> sh) & ((1 << P) - 1)
                assert got == int(nat[t, l]), (L, P, l, t)
                seen.add((lo, hi, sh))
        assert len(seen) == 7 * L                      # no two ids share their bits
    assert sk.codes_bytes(64, 10, 15) == -1 and sk.codes_bytes(64, 10, 32) == 2 * 20 * 64
    assert sk.codes_bytes(64, 8, 32) == 32 * 64 and sk.codes_bytes(64, 12, 32) == 32 * 64 * 2
    assert sk.codes_bytes(300, 2, 32) == 32 * 128 and sk.codes_bytes(128, 4, 32) == 32 * 64
    assert sk.codes_bytes(600, 2, 32) == 32 * 640 and sk.codes_bytes(7, 4, 16) == 16 * 16


def test_null_arguments_are_rejected_without_a_gpu():
    lib = sk.lib()
    assert lib.socket_create(None, None) == sk.EINVAL
    assert lib.socket_destroy(None) == sk.EINVAL
    assert lib.socket_hash_keys(None, None, None, None, None, None, 1, 1, None, None) == sk.EINVAL
    assert lib.socket_score(None, None, None, None, 0.5, None, None, None, 1, None, None) == sk.EINVAL
    assert lib.socket_topk_select(None, None, None, None, 1, None, None, None) == sk.EINVAL
    assert lib.socket_sparse_decode(None, None, None, None, None, None, None, 1, 1.0, 1, None, None) == sk.EINVAL
    assert lib.socket_dense_decode(None, None, None, None, None, None, 1, 1.0, 1, None, None) == sk.EINVAL
    assert lib.socket_value_norms(None, None, None, None, None, 1, 1, None, None) == sk.EINVAL
    assert lib.socket_set_forced_tokens(None, 4, 124) == sk.EINVAL
    assert lib.socket_score_keys_binned(None, None, None, None, None, 1, None, None) == sk.EINVAL
    assert lib.socket_topk_select_binned(None, None, None, None, 1, None, None, None) == sk.EINVAL
    assert lib.socket_reset(None, None) == sk.EINVAL
    assert lib.socket_bucket_probs(None, 1, None, None) == sk.EINVAL
    assert lib.socket_probe_stream_read(None, 16, None, None) == sk.EINVAL
    assert lib.socket_sparse_decode_noalloc(None, None, None, None, None, None, None, 1, 1.0, 1, None, None, None) == sk.EINVAL
    assert lib.socket_hard_hash(None, None, None, 1, None) == sk.EINVAL
    assert lib.socket_soft_hash(None, None, None, 0.5, 1, None) == sk.EINVAL
    assert lib.socket_score_keys(None, None, None, None, None, 1, None, None) == sk.EINVAL
    assert lib.socket_decode_step(None, None, None, None, None, None, 0.5, None, None, None, None, 1, 1.0, None,
                                  None, None, 1, None, None) == sk.EINVAL
    assert lib.socket_graph_begin(None) == sk.EINVAL
    assert lib.socket_scratch_bytes(None) == 0
