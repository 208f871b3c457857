"""ctypes binding of libsocket.so: the same calls as include/socket.h, taking torch tensors.

Argument marshalling only -- every step of the path runs in the library's HIP kernels.
PyTorch supplies device memory and the current stream.  If the shared library is missing
this module raises; there is no fallback implementation.
"""
import ctypes
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libsocket.so")

BF16, F32 = 0, 1
OK, EINVAL, EUNSUPPORTED, ENOMEM, EHIP, ELIMIT = 0, -1, -2, -3, -4, -5
NOALLOC_SCRATCH_BYTES = 4 * 1024 * 1024


class Params(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "d", "Hq", "Hkv", "L", "P", "kv_dtype", "max_batch", "max_n", "max_k", "page_size",
        "max_blocks_per_seq", "num_blocks")]


class SocketError(RuntimeError):
    def __init__(self, code, what):
        self.code = code
        super().__init__(f"{what}: {strerror(code)} ({code})")


_lib = None


def lib():
    """Load libsocket.so (built by `python -m paper_2602_06283_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2602_06283_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float
        L.socket_validate_params.argtypes = [ctypes.POINTER(Params)]
        L.socket_codes_per_token.argtypes = [i32]
        L.socket_code_position.argtypes = [i32, i32, i32]
        L.socket_codes_bytes.argtypes = [i32, i32, ctypes.c_int64]
        L.socket_codes_bytes.restype = ctypes.c_int64
        L.socket_code_location.argtypes = [i32, i32, i32, i32, ctypes.POINTER(ctypes.c_int64),
                                           ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(i32)]
        L.socket_create.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(Params)]
        L.socket_destroy.argtypes = [vp]
        L.socket_scratch_bytes.argtypes = [vp]
        L.socket_scratch_bytes.restype = ctypes.c_int64
        L.socket_hash_keys.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, vp, vp]
        L.socket_value_norms.argtypes = [vp, vp, vp, vp, vp, i32, i32, vp, vp]
        L.socket_set_forced_tokens.argtypes = [vp, i32, i32]
        L.socket_score.argtypes = [vp, vp, vp, vp, f32, vp, vp, vp, i32, vp, vp]
        L.socket_soft_hash.argtypes = [vp, vp, vp, f32, i32, vp]
        L.socket_hard_hash.argtypes = [vp, vp, vp, i32, vp]
        L.socket_score_keys.argtypes = [vp, vp, vp, vp, vp, i32, vp, vp]
        L.socket_topk_select.argtypes = [vp, vp, vp, vp, i32, vp, vp, vp]
        L.socket_score_keys_binned.argtypes = [vp, vp, vp, vp, vp, i32, vp, vp]
        L.socket_topk_select_binned.argtypes = [vp, vp, vp, vp, i32, vp, vp, vp]
        L.socket_reset.argtypes = [vp, vp]
        L.socket_bucket_probs.argtypes = [vp, i32, vp, vp]
        L.socket_probe_stream_read.argtypes = [vp, ctypes.c_int64, vp, vp]
        L.socket_sparse_decode.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, f32, i32, vp, vp]
        L.socket_sparse_decode_noalloc.argtypes = [ctypes.POINTER(Params), vp, vp, vp, vp, vp, vp, i32, f32, i32, vp,
                                                   vp, ctypes.POINTER(i32)]
        L.socket_dense_decode.argtypes = [vp, vp, vp, vp, vp, vp, i32, f32, i32, vp, vp]
        L.socket_decode_step.argtypes = [vp, vp, vp, vp, vp, vp, f32, vp, vp, vp, vp, i32, f32, vp, vp, vp,
                                         i32, vp, vp]
        L.socket_strerror.argtypes = [ctypes.c_int]
        L.socket_strerror.restype = ctypes.c_char_p
        L.socket_last_hip_error.argtypes = [vp]
        L.socket_graph_begin.argtypes = [vp]
        L.socket_graph_end.argtypes = [vp, ctypes.POINTER(vp)]
        L.socket_graph_launch.argtypes = [vp, vp]
        L.socket_graph_destroy.argtypes = [vp]
        _lib = L
    return _lib


EXPORTS = ("socket_validate_params", "socket_codes_per_token", "socket_code_position",
           "socket_codes_bytes", "socket_code_location",
           "socket_create", "socket_destroy", "socket_scratch_bytes", "socket_hash_keys",
           "socket_value_norms", "socket_set_forced_tokens",
           "socket_score", "socket_soft_hash", "socket_hard_hash", "socket_score_keys", "socket_score_keys_binned", "socket_topk_select", "socket_topk_select_binned", "socket_reset", "socket_bucket_probs", "socket_probe_stream_read", "socket_sparse_decode", "socket_sparse_decode_noalloc", "socket_dense_decode", "socket_decode_step", "socket_strerror",
           "socket_last_hip_error", "socket_graph_begin", "socket_graph_end",
           "socket_graph_launch", "socket_graph_destroy")


def strerror(code: int) -> str:
    return lib().socket_strerror(int(code)).decode()


def make_params(d, Hq, Hkv, L, P, kv_dtype, max_batch, max_n, max_k, page_size=0,
                max_blocks_per_seq=0, num_blocks=0) -> Params:
    return Params(d, Hq, Hkv, L, P, kv_dtype, max_batch, max_n, max_k, page_size,
                  max_blocks_per_seq, num_blocks)


def validate_params(p: Params) -> int:
    return lib().socket_validate_params(ctypes.byref(p))


def codes_per_token(L: int) -> int:
    return lib().socket_codes_per_token(L)


def code_position(L: int, l: int, t: int) -> int:
    return lib().socket_code_position(L, l, t)


def codes_bytes(L: int, P: int, tokens: int) -> int:
    return lib().socket_codes_bytes(L, P, tokens)


def code_location(L: int, P: int, l: int, t: int):
    """(lo_byte, hi_byte, hi_shift) of table l's bucket id of token t; see socket.h."""
    lo, hi, sh = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int32()
    rc = lib().socket_code_location(L, P, l, t, ctypes.byref(lo), ctypes.byref(hi), ctypes.byref(sh))
    if rc != OK:
        raise SocketError(rc, "socket_code_location")
    return lo.value, hi.value, sh.value


def _ptr(t):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensors only"
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


class Context:
    """socket_ctx with the four calls of the decode path as methods."""

    def __init__(self, params: Params):
        self.params = params
        self._h = ctypes.c_void_p()
        rc = lib().socket_create(ctypes.byref(self._h), ctypes.byref(params))
        if rc != OK:
            self._h = None
            raise SocketError(rc, "socket_create")

    def close(self):
        if getattr(self, "_h", None):
            lib().socket_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def scratch_bytes(self) -> int:
        return lib().socket_scratch_bytes(self._h)

    def _check(self, rc, what):
        if rc != OK:
            hip = lib().socket_last_hip_error(self._h)
            raise SocketError(rc, f"{what} (hip error {hip})")

    def hash_keys(self, K, proj, row_begin, row_count, batch, max_rows, codes, block_table=None,
                  stream=None):
        self._check(lib().socket_hash_keys(self._h, _ptr(K), _ptr(proj), _ptr(block_table),
                                           _ptr(row_begin), _ptr(row_count), batch, max_rows,
                                           _ptr(codes), _stream(stream)), "socket_hash_keys")

    def value_norms(self, V, row_begin, row_count, batch, max_rows, vnorm, block_table=None, stream=None):
        self._check(lib().socket_value_norms(self._h, _ptr(V), _ptr(block_table), _ptr(row_begin),
                                             _ptr(row_count), batch, max_rows, _ptr(vnorm),
                                             _stream(stream)), "socket_value_norms")

    def set_forced_tokens(self, n_sink, n_window):
        self._check(lib().socket_set_forced_tokens(self._h, int(n_sink), int(n_window)),
                    "socket_set_forced_tokens")

    def score(self, q, codes, proj, tau, seq_len, batch, scores, vnorm=None, block_table=None,
              stream=None):
        self._check(lib().socket_score(self._h, _ptr(q), _ptr(codes), _ptr(proj), float(tau),
                                       _ptr(vnorm), _ptr(block_table), _ptr(seq_len), batch,
                                       _ptr(scores), _stream(stream)), "socket_score")

    def soft_hash(self, q, proj, tau, batch, stream=None):
        self._check(lib().socket_soft_hash(self._h, _ptr(q), _ptr(proj), float(tau), batch,
                                           _stream(stream)), "socket_soft_hash")

    def hard_hash(self, q, proj, batch, stream=None):
        self._check(lib().socket_hard_hash(self._h, _ptr(q), _ptr(proj), batch, _stream(stream)),
                    "socket_hard_hash")

    def score_keys(self, codes, seq_len, batch, scores, vnorm=None, block_table=None, stream=None):
        self._check(lib().socket_score_keys(self._h, _ptr(codes), _ptr(vnorm), _ptr(block_table),
                                            _ptr(seq_len), batch, _ptr(scores), _stream(stream)),
                    "socket_score_keys")

    def score_keys_binned(self, codes, seq_len, batch, scores, vnorm=None, block_table=None, stream=None):
        self._check(lib().socket_score_keys_binned(self._h, _ptr(codes), _ptr(vnorm), _ptr(block_table),
                                                   _ptr(seq_len), batch, _ptr(scores), _stream(stream)),
                    "socket_score_keys_binned")

    def topk_select_binned(self, scores, seq_len, k, batch, idx, n_selected, stream=None):
        self._check(lib().socket_topk_select_binned(self._h, _ptr(scores), _ptr(seq_len), _ptr(k), batch,
                                                    _ptr(idx), _ptr(n_selected), _stream(stream)),
                    "socket_topk_select_binned")

    def reset(self, stream=None):
        self._check(lib().socket_reset(self._h, _stream(stream)), "socket_reset")

    def bucket_probs(self, batch, probs, stream=None):
        self._check(lib().socket_bucket_probs(self._h, batch, _ptr(probs), _stream(stream)), "socket_bucket_probs")

    def topk_select(self, scores, seq_len, k, batch, idx, n_selected, stream=None):
        self._check(lib().socket_topk_select(self._h, _ptr(scores), _ptr(seq_len), _ptr(k), batch,
                                             _ptr(idx), _ptr(n_selected), _stream(stream)),
                    "socket_topk_select")

    def sparse_decode(self, q, K, V, idx, n_selected, batch, scale, out, block_table=None,
                      stream=None):
        out_dtype = F32 if out.dtype == torch.float32 else BF16
        self._check(lib().socket_sparse_decode(self._h, _ptr(q), _ptr(K), _ptr(V), _ptr(idx),
                                               _ptr(n_selected), _ptr(block_table), batch,
                                               float(scale), out_dtype, _ptr(out), _stream(stream)),
                    "socket_sparse_decode")

    def dense_decode(self, q, K, V, seq_len, batch, scale, out, block_table=None, stream=None):
        out_dtype = F32 if out.dtype == torch.float32 else BF16
        self._check(lib().socket_dense_decode(self._h, _ptr(q), _ptr(K), _ptr(V), _ptr(block_table),
                                              _ptr(seq_len), batch, float(scale), out_dtype, _ptr(out),
                                              _stream(stream)), "socket_dense_decode")

    def decode_step(self, q, K, V, codes, proj, tau, pos, k, batch, scale, scores, idx, n_selected, out,
                    vnorm=None, block_table=None, stream=None):
        out_dtype = F32 if out.dtype == torch.float32 else BF16
        self._check(lib().socket_decode_step(self._h, _ptr(q), _ptr(K), _ptr(V), _ptr(codes), _ptr(proj),
                                             float(tau), _ptr(vnorm), _ptr(block_table), _ptr(pos),
                                             _ptr(k), batch, float(scale), _ptr(scores), _ptr(idx),
                                             _ptr(n_selected), out_dtype, _ptr(out), _stream(stream)),
                    "socket_decode_step")


def sparse_decode_noalloc(params: Params, q, K, V, idx, n_selected, batch, scale, out, block_table=None,
                          stream=None):
    """socket_sparse_decode_noalloc: no context, no allocation (see socket.h)."""
    out_dtype = F32 if out.dtype == torch.float32 else BF16
    hip = ctypes.c_int32(0)
    rc = lib().socket_sparse_decode_noalloc(ctypes.byref(params), _ptr(q), _ptr(K), _ptr(V), _ptr(idx),
                                            _ptr(n_selected), _ptr(block_table), batch, float(scale),
                                            out_dtype, _ptr(out), _stream(stream), ctypes.byref(hip))
    if rc != OK:
        raise SocketError(rc, f"socket_sparse_decode_noalloc (hip error {hip.value})")


def probe_stream_read(buf, sink, stream=None):
    """socket_probe_stream_read over the whole tensor `buf` (measurement aid, see socket.h)."""
    rc = lib().socket_probe_stream_read(_ptr(buf), buf.numel() * buf.element_size(), _ptr(sink), _stream(stream))
    if rc != OK:
        raise SocketError(rc, "socket_probe_stream_read")


class Graph:
    """A captured chain of library calls: `with Graph.capture(stream) as g: ...; g.launch()`."""

    def __init__(self, stream):
        self.stream = stream
        self._h = ctypes.c_void_p()

    @classmethod
    def capture(cls, stream):
        return cls(stream)

    def __enter__(self):
        rc = lib().socket_graph_begin(ctypes.c_void_p(self.stream.cuda_stream))
        if rc != OK:
            raise SocketError(rc, "socket_graph_begin")
        return self

    def __exit__(self, et, ev, tb):
        rc = lib().socket_graph_end(ctypes.c_void_p(self.stream.cuda_stream), ctypes.byref(self._h))
        if rc != OK and et is None:
            raise SocketError(rc, "socket_graph_end")
        return False

    def launch(self, stream=None):
        s = stream if stream is not None else self.stream
        rc = lib().socket_graph_launch(self._h, ctypes.c_void_p(s.cuda_stream))
        if rc != OK:
            raise SocketError(rc, "socket_graph_launch")

    def close(self):
        if self._h:
            lib().socket_graph_destroy(self._h)
            self._h = ctypes.c_void_p()
