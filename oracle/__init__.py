"""CPU oracle for the AttnCache hot path -- TEST INFRASTRUCTURE ONLY.

A ctypes front-end to ``attncache_oracle.c``.  Only ``tests/``, the smoke check
and the benchmark's ``cpu_baseline`` leg import this package; the GPU library
and its Python binding never do, and this package imports nothing of theirs.

All array arguments are numpy arrays.  Floating-point inputs are converted to
float32 here; that conversion is exact for the fp16 / bf16 / fp32 values the
hot path stores, and the C code widens every element to double before use.
"""
import ctypes
import os

import numpy as np

from . import build as _build

METRIC_IP = 0
METRIC_L2 = 1
ROUND_F32 = 0
ROUND_BF16 = 1

_lib = None


def lib():
    """Load (building first if needed) the oracle shared library."""
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = ctypes.CDLL(path)
        i32, i64, f32, f64, vp = (ctypes.c_int32, ctypes.c_int64, ctypes.c_float,
                                  ctypes.c_double, ctypes.c_void_p)
        L.oracle_search.restype = i32
        L.oracle_search.argtypes = [vp, vp, vp, i32, i32, i32, i32, f32, i32, vp, vp, vp]
        L.oracle_apply.restype = i32
        L.oracle_apply.argtypes = [vp, vp, vp, vp] + [i32] * 9
        L.oracle_attention_exact.restype = i32
        L.oracle_attention_exact.argtypes = [vp, vp, vp, vp, vp, vp, vp] + [i32] * 6 + [f64]
        L.oracle_round_maps.restype = i32
        L.oracle_round_maps.argtypes = [vp, vp, i64, i32]
        L.oracle_project.restype = i32
        L.oracle_project.argtypes = [vp] * 7 + [i32] * 6
        L.oracle_threads.restype = i32
        L.oracle_threads.argtypes = []
        _lib = L
    return _lib


def _f32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float32))


def _i32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check(rc, what):
    if rc != 0:
        raise RuntimeError(f"{what} failed with oracle status {rc}")


def threads() -> int:
    return int(lib().oracle_threads())


def search(q, emb, k=1, theta=0.0, metric=METRIC_IP, map_of=None):
    """Exact top-k search.  Returns (idx[B,k] int32, score[B,k] float32, hit[B] int32)."""
    q, emb = _f32(q), _f32(emb)
    B, E = q.shape
    N, E2 = emb.shape
    if E != E2:
        raise ValueError("embedding dims differ")
    mo = None if map_of is None else _i32(map_of)
    idx = np.empty((B, k), np.int32)
    score = np.empty((B, k), np.float32)
    hit = np.empty((B,), np.int32)
    _check(lib().oracle_search(_p(q), _p(emb), _p(mo), B, N, E, k, float(theta), metric,
                               _p(idx), _p(score), _p(hit)), "oracle_search")
    return idx, score, hit


def apply(maps, hit, V, layer_begin=0, out=None):
    """Reuse branch.  maps[M,L,Hq,S,S], hit[B], V[B,Lc,Hkv,S,D] -> O[B,Lc,Hq,S,D] float64.

    Rows of ``out`` (default: zeros) belonging to misses (hit == -1) are left as they are.
    """
    maps, V, hit = _f32(maps), _f32(V), _i32(hit)
    M, L, Hq, S, S2 = maps.shape
    B, Lc, Hkv, S3, D = V.shape
    if S != S2 or S != S3:
        raise ValueError("sequence lengths differ")
    if out is None:
        out = np.zeros((B, Lc, Hq, S, D), np.float64)
    assert out.dtype == np.float64 and out.flags.c_contiguous and out.shape == (B, Lc, Hq, S, D)
    _check(lib().oracle_apply(_p(maps), _p(hit), _p(V), _p(out), B, M, L, layer_begin, Lc,
                              Hq, Hkv, S, D), "oracle_apply")
    return out


def attention_exact(Q, K, V, causal=True, scale=0.0, row_sel=None, return_map=False, out=None,
                    key_len=None):
    """Recompute branch.  Q[B,Hq,S,D], K,V[B,Hkv,S,D] -> O[B,Hq,S,D] float64 (and P[B,Hq,S,S]).

    key_len[B] (optional): real tokens per sentence of a right-padded batch; later keys are hidden.
    """
    Q, K, V = _f32(Q), _f32(K), _f32(V)
    B, Hq, S, D = Q.shape
    Bk, Hkv, Sk, Dk = K.shape
    if (Bk, Sk, Dk) != (B, S, D) or V.shape != K.shape:
        raise ValueError("Q/K/V shapes disagree")
    if out is None:
        out = np.zeros((B, Hq, S, D), np.float64)
    P = np.zeros((B, Hq, S, S), np.float64) if return_map else None
    rs = None if row_sel is None else _i32(row_sel)
    kl = None if key_len is None else _i32(key_len)
    if kl is not None and kl.shape != (B,):
        raise ValueError("key_len must have one entry per batch item")
    _check(lib().oracle_attention_exact(_p(Q), _p(K), _p(V), _p(out), _p(P), _p(rs), _p(kl), B, Hq, Hkv,
                                        S, D, int(bool(causal)), float(scale)),
           "oracle_attention_exact")
    return (out, P) if return_map else out


def round_maps(P, kind=ROUND_BF16):
    """Storage rounding of computed maps (float64 in, float32 holding the rounded values out)."""
    P = np.ascontiguousarray(np.asarray(P, dtype=np.float64))
    out = np.empty(P.shape, np.float32)
    _check(lib().oracle_round_maps(_p(P), _p(out), P.size, kind), "oracle_round_maps")
    return out


def project(h, W1, b1, W2, b2, seq_len=None, normalize=True):
    """Feature projector.  h[B,S,dm], W1[hid,dm], b1[hid]|None, W2[E,hid], b2[E]|None -> f[B,E] float64."""
    h, W1, W2 = _f32(h), _f32(W1), _f32(W2)
    B, S, dm = h.shape
    hid, dm2 = W1.shape
    E, hid2 = W2.shape
    if dm != dm2 or hid != hid2:
        raise ValueError("weight shapes disagree with the input")
    b1 = None if b1 is None else _f32(b1)
    b2 = None if b2 is None else _f32(b2)
    if (b1 is not None and b1.shape != (hid,)) or (b2 is not None and b2.shape != (E,)):
        raise ValueError("bias shapes disagree with the weights")
    sl = None if seq_len is None else _i32(seq_len)
    out = np.empty((B, E), np.float64)
    _check(lib().oracle_project(_p(h), _p(sl), _p(W1), _p(b1), _p(W2), _p(b2), _p(out),
                                B, S, dm, hid, E, int(bool(normalize))), "oracle_project")
    return out
