"""CPU oracle for the SOCKET decode path (test infrastructure only).

Import this from tests, the smoke check and the benchmark's CPU-baseline leg.
The GPU library never imports it.
"""
from .socket_oracle import (  # noqa: F401
    hash_keys, soft_probs, score, hard_score, topk, sparse_decode, dense_decode,
    value_norms, force_tokens, num_threads, precision, jaccard, ndcg,
)
