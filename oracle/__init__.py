"""CPU oracle for one GPU's share of ESP attention -- TEST INFRASTRUCTURE ONLY.

Plain fp64 statements of what the hot path computes (LoongServe, arXiv
2404.09526: partial attention of Sec. 2.3 / Fig. 1, distributed decoding of
Sec. 4.2 / Fig. 8, token-granular KV pool of Sec. 6, selective retention of
Sec. 4.1 / Fig. 7).  Only tests, the smoke check and the benchmark's
cpu_baseline leg may import this package; it shares nothing with the HIP path
and does not import it.

Two independent statements live here:
  * the C library ``esp_oracle.c`` (row-by-row, three passes), wrapped below;
  * ``brute_force_attention`` (dense score matrix in numpy), which exists only
    to pin the C routine on tiny inputs.
Pinning status: every function below is pinned by tests/test_oracle_pins.py
(brute force, also on every request's slice of a packed var-len shard through the
per-sample key-row range; a library attention routine; closed forms; partition and
permutation invariance).  The paper prints no numeric worked example, so no
paper-printed value is among the pins.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "esp_oracle.c")
_LIB = os.path.join(_HERE, "libesp_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile esp_oracle.c with gcc (-O2 -fopenmp) into libesp_oracle.so."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        vp, i64, f64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_double, ctypes.c_int
        L.oracle_partial_attn.argtypes = [vp] * 5 + [i64, i64, i64, f64, i32, i64] + [vp] * 6
        L.oracle_partial_attn.restype = i32
        L.oracle_partial_attn_decode.argtypes = [vp] * 5 + [i64, i64, i64, f64, i64] + [vp] * 4
        L.oracle_partial_attn_decode.restype = i32
        L.oracle_merge_partials.argtypes = [vp, vp, i64, i64, i64, vp, vp]
        L.oracle_merge_partials.restype = i32
        L.oracle_kv_append.argtypes = [vp, vp, vp, i64, i64, i64, vp, vp]
        L.oracle_kv_append.restype = i32
        L.oracle_num_threads.argtypes = []
        L.oracle_num_threads.restype = i32
        _lib = L
    return _lib


def _p(a: np.ndarray):
    return ctypes.c_void_p(a.ctypes.data)


def _bits(a, name) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint16:
        raise TypeError(f"{name}: expected bf16 bit patterns as uint16, got {a.dtype}")
    return a


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _i64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int64)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact value of bf16 bit patterns (uint16) as float64."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def partial_attn(q, k, v, q_pos, kv_pos, scale, causal, rows, heads, kv_lo=None, kv_hi=None):
    """Partial attention (Sec. 2.3 / Fig. 1) for sampled (row, head) pairs.

    q [Tq,Hq,D], k/v [Tkv,Hkv,D] as uint16 bf16 bits; positions int32.  Sample i
    attends query (rows[i], heads[i]) to key rows [kv_lo[i], kv_hi[i]) (default:
    the whole shard).  Returns (O [n,D] float64, LSE [n] float64).
    """
    q, k, v = _bits(q, "q"), _bits(k, "k"), _bits(v, "v")
    Tq, Hq, D = q.shape
    Tkv, Hkv, _ = k.shape
    assert v.shape == k.shape and k.shape[2] == D
    q_pos, kv_pos = _i32(q_pos), _i32(kv_pos)
    assert q_pos.shape == (Tq,) and kv_pos.shape == (Tkv,)
    rows, heads = _i64(rows), _i64(heads)
    n = rows.shape[0]
    kv_lo = np.zeros(n, np.int64) if kv_lo is None else _i64(kv_lo)
    kv_hi = np.full(n, Tkv, np.int64) if kv_hi is None else _i64(kv_hi)
    assert heads.shape == (n,) and kv_lo.shape == (n,) and kv_hi.shape == (n,)
    assert n == 0 or (rows.min() >= 0 and rows.max() < Tq and heads.min() >= 0 and heads.max() < Hq)
    assert n == 0 or (kv_lo.min() >= 0 and kv_hi.max() <= Tkv and (kv_lo <= kv_hi).all())
    O = np.zeros((n, D), np.float64)
    LSE = np.zeros(n, np.float64)
    rc = _load().oracle_partial_attn(_p(q), _p(k), _p(v), _p(q_pos), _p(kv_pos), Hq, Hkv, D,
                                     float(scale), int(bool(causal)), n, _p(rows), _p(heads),
                                     _p(kv_lo), _p(kv_hi), _p(O), _p(LSE))
    if rc != 0:
        raise RuntimeError("oracle_partial_attn failed")
    return O, LSE


def partial_attn_all(q, k, v, q_pos, kv_pos, scale, causal):
    """Partial attention for every (row, head): (O [Tq,Hq,D], LSE [Tq,Hq])."""
    Tq, Hq, D = q.shape
    rows = np.repeat(np.arange(Tq, dtype=np.int64), Hq)
    heads = np.tile(np.arange(Hq, dtype=np.int64), Tq)
    O, LSE = partial_attn(q, k, v, q_pos, kv_pos, scale, causal, rows, heads)
    return O.reshape(Tq, Hq, D), LSE.reshape(Tq, Hq)


def partial_attn_decode(q, k_pool, v_pool, slot_idx, seq_offsets, scale, reqs, heads):
    """Decode partial attention (Sec. 4.2 / Fig. 8) for sampled (request, head) pairs.

    q [B,Hq,D], pools [S,Hkv,D] as uint16 bf16 bits.  Request b attends to pool rows
    slot_idx[seq_offsets[b]:seq_offsets[b+1]].  Returns (O [n,D], LSE [n]) float64.
    """
    q, k_pool, v_pool = _bits(q, "q"), _bits(k_pool, "k_pool"), _bits(v_pool, "v_pool")
    B, Hq, D = q.shape
    S, Hkv, _ = k_pool.shape
    assert v_pool.shape == k_pool.shape and k_pool.shape[2] == D
    slot_idx, seq_offsets = _i32(slot_idx), _i32(seq_offsets)
    assert seq_offsets.shape == (B + 1,) and seq_offsets[-1] <= slot_idx.shape[0]
    assert slot_idx.size == 0 or (slot_idx.min() >= 0 and slot_idx.max() < S)
    reqs, heads = _i64(reqs), _i64(heads)
    n = reqs.shape[0]
    assert n == 0 or (reqs.min() >= 0 and reqs.max() < B and heads.min() >= 0 and heads.max() < Hq)
    O = np.zeros((n, D), np.float64)
    LSE = np.zeros(n, np.float64)
    rc = _load().oracle_partial_attn_decode(_p(q), _p(k_pool), _p(v_pool), _p(slot_idx),
                                            _p(seq_offsets), Hq, Hkv, D, float(scale), n,
                                            _p(reqs), _p(heads), _p(O), _p(LSE))
    if rc != 0:
        raise RuntimeError("oracle_partial_attn_decode failed")
    return O, LSE


def partial_attn_decode_all(q, k_pool, v_pool, slot_idx, seq_offsets, scale):
    B, Hq, D = q.shape
    reqs = np.repeat(np.arange(B, dtype=np.int64), Hq)
    heads = np.tile(np.arange(Hq, dtype=np.int64), B)
    O, LSE = partial_attn_decode(q, k_pool, v_pool, slot_idx, seq_offsets, scale, reqs, heads)
    return O.reshape(B, Hq, D), LSE.reshape(B, Hq)


def merge_partials(O_parts, LSE_parts):
    """Log-sum-exp weighted combination of P partials (Sec. 2.3, Sec. 4.2).

    O_parts [P, ..., D], LSE_parts [P, ...] float64 values (callers convert bf16
    partials with bf16_bits_to_f64 first).  Returns (O [..., D], LSE [...]).
    """
    O_parts = np.ascontiguousarray(O_parts, dtype=np.float64)
    LSE_parts = np.ascontiguousarray(LSE_parts, dtype=np.float64)
    P, D = O_parts.shape[0], O_parts.shape[-1]
    lead = O_parts.shape[1:-1]
    assert LSE_parts.shape == (P,) + lead
    n = int(np.prod(lead)) if lead else 1
    O = np.zeros((n, D), np.float64)
    LSE = np.zeros(n, np.float64)
    rc = _load().oracle_merge_partials(_p(O_parts), _p(LSE_parts), P, n, D, _p(O), _p(LSE))
    if rc != 0:
        raise RuntimeError("oracle_merge_partials failed")
    return O.reshape(lead + (D,)), LSE.reshape(lead)


def kv_append(k, v, slot_idx, k_pool, v_pool):
    """Scatter rows into pool slots in place (Sec. 4.1 / Fig. 7); slot < 0 skips the row."""
    k, v = _bits(k, "k"), _bits(v, "v")
    for pool in (k_pool, v_pool):
        if pool.dtype != np.uint16 or not pool.flags.c_contiguous or not pool.flags.writeable:
            raise TypeError("pools must be writable C-contiguous uint16 arrays")
    T = k.shape[0]
    row = int(np.prod(k.shape[1:]))
    assert v.shape == k.shape and k_pool.shape == v_pool.shape
    assert int(np.prod(k_pool.shape[1:])) == row
    slot_idx = _i32(slot_idx)
    assert slot_idx.shape == (T,)
    rc = _load().oracle_kv_append(_p(k), _p(v), _p(slot_idx), T, row, k_pool.shape[0],
                                  _p(k_pool), _p(v_pool))
    if rc != 0:
        raise ValueError("oracle_kv_append: slot out of range")


def kv_gather(k_pool, v_pool, slot_idx):
    """Rows of the pool in the order of a slot list: the dense view of the key-value rows a request keeps in the
    token-granular pool (Sec. 4.1 / Fig. 7; Sec. 6); the inverse of kv_append.  A slot that is negative or not below
    the number of slots gives a row of zeros.  Returns (k, v) as uint16 [T, ...]."""
    k_pool, v_pool = _bits(k_pool, "k_pool"), _bits(v_pool, "v_pool")
    assert k_pool.shape == v_pool.shape
    slot_idx = _i32(slot_idx)
    assert slot_idx.ndim == 1
    k = np.zeros((slot_idx.shape[0],) + k_pool.shape[1:], np.uint16)
    v = np.zeros_like(k)
    for t in range(slot_idx.shape[0]):
        s = int(slot_idx[t])
        if 0 <= s < k_pool.shape[0]:
            k[t] = k_pool[s]
            v[t] = v_pool[s]
    return k, v


def brute_force_attention(q, k, v, q_pos, kv_pos, scale, causal):
    """Dense-matrix softmax attention in numpy fp64, for pinning on tiny inputs only.

    Written differently from the C routine on purpose: the whole masked score
    matrix, a row softmax, one matrix product, and log-sum-exp from the matrix.
    q [Tq,Hq,D], k/v [Tkv,Hkv,D] uint16 bf16 bits.  Returns (O [Tq,Hq,D], LSE [Tq,Hq]).
    """
    qf, kf, vf = bf16_bits_to_f64(q), bf16_bits_to_f64(k), bf16_bits_to_f64(v)
    Tq, Hq, D = qf.shape
    Tkv, Hkv, _ = kf.shape
    G = Hq // Hkv
    O = np.zeros((Tq, Hq, D))
    LSE = np.full((Tq, Hq), -np.inf)
    hidden = np.zeros((Tq, Tkv), bool)
    if causal:
        hidden = np.asarray(kv_pos)[None, :] > np.asarray(q_pos)[:, None]
    for h in range(Hq):
        S = scale * (qf[:, h, :] @ kf[:, h // G, :].T)
        S[hidden] = -np.inf
        with np.errstate(invalid="ignore", divide="ignore"):
            E = np.exp(S)                      # tiny inputs: no overflow concern
            Z = E.sum(axis=1)
            Pm = np.where(Z[:, None] > 0, E / Z[:, None], 0.0)
            LSE[:, h] = np.log(Z)
        O[:, h, :] = Pm @ vf[:, h // G, :]
    return O, LSE
