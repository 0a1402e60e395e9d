"""fp64 reference attention over the logical sequence (test infrastructure only).

What is computed (paper Sec. 4.2: each of the P new tokens of a request interacts with its
C pre-existing context tokens and with the earlier tokens of its own chunk; Sec. 2 on the
KV cache; chunked prefill paragraph of Sec. 4.2): for a request with prior context C and q
new tokens, new token i sits at absolute position p = C + i and, for query head h with kv
head g = h // (Hq // Hkv),

    s_j = scale * <q[i, h], K[j, g]>          j = 0 .. p
    w_j = exp(s_j - max s) / sum_j exp(s_j - max s)
    out[i, h] = sum_j w_j * V[j, g]

The arithmetic is in ``cs_oracle.c`` (plain loops, double precision).  The oracle never
sees pages or block tables.
"""
import ctypes

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(_build.build())
        lib.cs_ref_attention_seq.restype = ctypes.c_int
        lib.cs_ref_attention_seq.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32,
            ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_double,
            ctypes.c_void_p, ctypes.c_void_p,
        ]
        lib.cs_ref_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    """Threads the C loops use (OpenMP default for this process)."""
    return int(_load().cs_ref_num_threads())


def attention_rows(q, positions, k, v, scale, return_weight_sums=False):
    """Attention of arbitrary query rows of ONE request.

    q [nq, Hq, D], positions [nq] (absolute position of each row; row attends keys
    0..position), k / v [n, Hkv, D] logical keys / values (n > max position).  Inputs may be
    any float dtype; they are used as float32 (exact for bf16-representable values).
    Returns float64 [nq, Hq, D] (and the per-row sum of softmax weights if asked).
    """
    q = np.ascontiguousarray(q, dtype=np.float32)
    k = np.ascontiguousarray(k, dtype=np.float32)
    v = np.ascontiguousarray(v, dtype=np.float32)
    positions = np.ascontiguousarray(positions, dtype=np.int32)
    nq, Hq, D = q.shape
    n, Hkv, Dk = k.shape
    assert v.shape == k.shape and Dk == D and positions.shape == (nq,)
    out = np.empty((nq, Hq, D), dtype=np.float64)
    wsum = np.empty((nq, Hq), dtype=np.float64)
    if nq == 0:
        return (out, wsum) if return_weight_sums else out
    rc = _load().cs_ref_attention_seq(
        q.ctypes.data, positions.ctypes.data, nq, k.ctypes.data, v.ctypes.data, n,
        Hq, Hkv, D, float(scale), out.ctypes.data, wsum.ctypes.data)
    if rc != 0:
        raise ValueError("cs_ref_attention_seq failed with code %d" % rc)
    return (out, wsum) if return_weight_sums else out


def attention_chunk(q, k, v, ctx_len, scale, return_weight_sums=False):
    """One request's step: q [q_len, Hq, D] new tokens on top of ``ctx_len`` prior tokens.

    k / v hold at least ctx_len + q_len logical rows (the new tokens' K/V already appended).
    A decode token is the case q_len == 1.
    """
    q_len = q.shape[0]
    positions = np.arange(ctx_len, ctx_len + q_len, dtype=np.int32)
    return attention_rows(q, positions, k, v, scale, return_weight_sums)


def attention_batch(q, seq_k, seq_v, ctx_lens, q_lens, scale):
    """A mixed batch: q [T, Hq, D] packed in sequence order; seq_k / seq_v are lists of the
    requests' logical K / V (each with ctx + q_len rows).  Returns float64 [T, Hq, D]."""
    q = np.asarray(q)
    out = np.empty(q.shape, dtype=np.float64)
    t = 0
    for s, (c, ql) in enumerate(zip(ctx_lens, q_lens)):
        c, ql = int(c), int(ql)
        if ql:
            out[t:t + ql] = attention_chunk(q[t:t + ql], seq_k[s], seq_v[s], c, scale)
        t += ql
    assert t == q.shape[0]
    return out
