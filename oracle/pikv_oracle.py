"""ctypes front-end of the CPU oracle (``pikv_oracle.c``).

Test infrastructure only: the test-suite, the smoke check and the benchmark's
``cpu_baseline`` leg call it; the product package never does.  Arrays are numpy, on the
host; bfloat16 data travels as ``uint16`` bit patterns (``dtype='bf16'``).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pikv_oracle.c")
_LIB = os.path.join(_HERE, "libpikv_oracle.so")

F32, BF16 = 0, 1
COMBINE_LSE, COMBINE_LOCAL = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, -O2, OpenMP over independent units)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        # PIKV_ORACLE_LIB lets the mutation test load a deliberately broken build
        _lib = C.CDLL(os.environ.get("PIKV_ORACLE_LIB") or build())
        for name in ("pikv_oracle_route", "pikv_oracle_attend", "pikv_oracle_evict",
                     "pikv_oracle_append", "pikv_oracle_router_penalty", "pikv_oracle_compress",
                     "pikv_oracle_policy_stamp", "pikv_oracle_policy_access",
                     "pikv_oracle_policy_utility", "pikv_oracle_policy_compact", "pikv_oracle_route_round_robin"):
            getattr(_lib, name).restype = C.c_int
    return _lib


def _dt(dtype) -> int:
    return {"f32": F32, "bf16": BF16, F32: F32, BF16: BF16}[dtype]


def _np_dtype(dtype):
    return np.float32 if _dt(dtype) == F32 else np.uint16


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _chk(a, dtype, name):
    if a is None:
        return None
    if not isinstance(a, np.ndarray) or a.dtype != dtype or not a.flags["C_CONTIGUOUS"]:
        raise TypeError("%s must be a C-contiguous numpy array of %s" % (name, dtype))
    return a


def _ptr_table(shards):
    """list of numpy arrays -> (ctypes void* array, keep-alive)."""
    arr = (C.c_void_p * len(shards))()
    for i, s in enumerate(shards):
        arr[i] = s.ctypes.data
    return arr


def route(x, W_r, k, bias=None, dtype="f32", want_logits=False):
    """x [rows,d_r], W_r [d_r,E] -> idx int32 [rows,k], gates f32 [rows,k], probs f32 [rows,E]."""
    nd = _np_dtype(dtype)
    x = _chk(x, nd, "x")
    W_r = _chk(W_r, nd, "W_r")
    rows, d_r = x.shape
    E = W_r.shape[1]
    assert W_r.shape[0] == d_r
    bias = _chk(bias, np.float32, "bias")
    idx = np.zeros((rows, k), np.int32)
    gates = np.zeros((rows, k), np.float32)
    probs = np.zeros((rows, E), np.float32)
    logits = np.zeros((rows, E), np.float64)
    rc = lib().pikv_oracle_route(_ptr(x), _ptr(W_r), _ptr(bias), rows, d_r, E, k, _dt(dtype),
                                 _ptr(idx), _ptr(gates), _ptr(probs), _ptr(logits))
    if rc:
        raise ValueError("pikv_oracle_route failed: %d" % rc)
    if want_logits:
        return idx, gates, probs, logits
    return idx, gates, probs


def attend(q, K_shards, V_shards, n_valid, topk_idx, gates, *, Hkv, E, S, dtype="f32",
           rank=0, U_K=None, U_V=None, V_bias=None, combine=COMBINE_LSE, scale=0.0, stride_h=None,
           stride_s=None, utility=None, decay=1.0, want_prob=False):
    """One decode step of routed attention (+ optional in-place utility update).

    q [B,Hq,D]; K_shards/V_shards: list of B*E arrays, each [Hkv,S,w] (w = D or rank);
    n_valid int32 [B,E]; topk_idx int32 [R,k] with R = B (per-token) or B*Hq (per-head);
    gates f32 [R,k] or None.  Returns dict(y, row_max, row_norm[, prob]).
    """
    nd = _np_dtype(dtype)
    q = _chk(q, nd, "q")
    B, Hq, D = q.shape
    w = rank if rank else D
    if stride_s is None:
        stride_s = w
    if stride_h is None:
        stride_h = S * stride_s
    assert len(K_shards) == B * E and len(V_shards) == B * E
    for s in list(K_shards) + list(V_shards):
        _chk(s, nd, "shard")
    n_valid = _chk(n_valid, np.int32, "n_valid")
    topk_idx = _chk(topk_idx, np.int32, "topk_idx")
    gates = _chk(gates, np.float32, "gates")
    R, k = topk_idx.shape
    assert R in (B, B * Hq)
    rr = 1 if R == B else Hq
    U_K = _chk(U_K, nd, "U_K")
    U_V = _chk(U_V, nd, "U_V")
    V_bias = _chk(V_bias, nd, "V_bias")
    utility = _chk(utility, np.float32, "utility")
    y = np.zeros((B, Hq, D), np.float32)
    row_max = np.zeros((B, Hq), np.float32)
    row_norm = np.zeros((B, Hq), np.float32)
    prob = np.zeros((B, Hq, k, S), np.float64) if want_prob else None
    kt, vt = _ptr_table(K_shards), _ptr_table(V_shards)
    rc = lib().pikv_oracle_attend(
        B, Hq, Hkv, D, E, S, rank, _dt(dtype), C.c_int64(stride_h), C.c_int64(stride_s), rr,
        _ptr(q), kt, vt, _ptr(U_K), _ptr(U_V), _ptr(V_bias), _ptr(n_valid), _ptr(topk_idx), _ptr(gates), k,
        combine, C.c_double(scale), _ptr(y), _ptr(row_max), _ptr(row_norm), _ptr(prob),
        C.c_double(decay), _ptr(utility))
    if rc:
        raise ValueError("pikv_oracle_attend failed: %d" % rc)
    out = {"y": y, "row_max": row_max, "row_norm": row_norm}
    if want_prob:
        out["prob"] = prob
    return out


def evict(utility, n_valid, capacity, *, shard_mask=None, max_evict=None, compact=False,
          K_shards=None, V_shards=None, Hkv=0, width=0, dtype="f32", stride_h=None,
          stride_s=None):
    """In place on utility / n_valid (/ shards when compact).  Returns (evicted_idx, evicted_cnt)."""
    utility = _chk(utility, np.float32, "utility")
    n_valid = _chk(n_valid, np.int32, "n_valid")
    B, E, S = utility.shape
    shard_mask = _chk(shard_mask, np.int32, "shard_mask")
    if max_evict is None:
        max_evict = max(0, S - capacity)
    if stride_s is None:
        stride_s = width
    if stride_h is None:
        stride_h = S * stride_s
    idx = np.full((B, E, max_evict), -1, np.int32)
    cnt = np.zeros((B, E), np.int32)
    kt = _ptr_table(K_shards) if K_shards is not None else None
    vt = _ptr_table(V_shards) if V_shards is not None else None
    rc = lib().pikv_oracle_evict(B, E, S, Hkv, width, _dt(dtype), C.c_int64(stride_h),
                                 C.c_int64(stride_s), _ptr(utility), _ptr(n_valid), capacity,
                                 _ptr(shard_mask), _ptr(idx), _ptr(cnt), max_evict,
                                 1 if compact else 0, kt, vt)
    if rc:
        raise ValueError("pikv_oracle_evict failed: %d" % rc)
    return idx, cnt


def append(K_new, V_new, topk_idx, K_shards, V_shards, utility, n_valid, *, dtype="f32",
           reuse_idx=None, reuse_cnt=None, stride_h=None, stride_s=None):
    """In place on the shards, utility and n_valid.  K_new/V_new [B,Hkv,w]; topk_idx [B,k]."""
    nd = _np_dtype(dtype)
    K_new = _chk(K_new, nd, "K_new")
    V_new = _chk(V_new, nd, "V_new")
    B, Hkv, width = K_new.shape
    _, E, S = utility.shape
    topk_idx = _chk(topk_idx, np.int32, "topk_idx")
    k = topk_idx.shape[1]
    if stride_s is None:
        stride_s = width
    if stride_h is None:
        stride_h = S * stride_s
    max_evict = 0
    if reuse_idx is not None:
        reuse_idx = _chk(reuse_idx, np.int32, "reuse_idx")
        reuse_cnt = _chk(reuse_cnt, np.int32, "reuse_cnt")
        max_evict = reuse_idx.shape[2]
    kt, vt = _ptr_table(K_shards), _ptr_table(V_shards)
    rc = lib().pikv_oracle_append(B, E, S, Hkv, width, _dt(dtype), C.c_int64(stride_h),
                                  C.c_int64(stride_s), _ptr(K_new), _ptr(V_new), _ptr(topk_idx),
                                  k, _ptr(reuse_idx), _ptr(reuse_cnt), max_evict, kt, vt,
                                  _ptr(_chk(utility, np.float32, "utility")),
                                  _ptr(_chk(n_valid, np.int32, "n_valid")))
    if rc:
        raise ValueError("pikv_oracle_append failed: %d" % rc)


LB, CACHE_AWARE, ENTROPY = 0, 1, 2


def router_penalty(mode, topk_idx, load, coef, miss=None):
    """In place on load [E] int32 (absorbs topk_idx [rows,k]).  Returns bias f32 [E]."""
    topk_idx = _chk(topk_idx, np.int32, "topk_idx")
    load = _chk(load, np.int32, "load")
    miss = _chk(miss, np.int32, "miss")
    rows, k = topk_idx.shape
    E = load.shape[0]
    bias = np.zeros(E, np.float32)
    rc = lib().pikv_oracle_router_penalty(mode, _ptr(topk_idx), rows, k, E, _ptr(load), _ptr(miss),
                                          C.c_double(coef), _ptr(bias))
    if rc:
        raise ValueError("pikv_oracle_router_penalty failed: %d" % rc)
    return bias


def compress(x, W_enc, dtype="f32"):
    """x [B,Hkv,D], W_enc [Hkv,rank,D] (storage dtype) -> codes [B,Hkv,rank] (storage dtype)."""
    nd = _np_dtype(dtype)
    x = _chk(x, nd, "x")
    W_enc = _chk(W_enc, nd, "W_enc")
    B, Hkv, D = x.shape
    rank = W_enc.shape[1]
    codes = np.zeros((B, Hkv, rank), nd)
    rc = lib().pikv_oracle_compress(B, Hkv, D, rank, _dt(dtype), _ptr(x), _ptr(W_enc), _ptr(codes))
    if rc:
        raise ValueError("pikv_oracle_compress failed: %d" % rc)
    return codes


POLICY_H2O, POLICY_SL, POLICY_LRU, POLICY_LRU_PLUS = 0, 1, 2, 3


def policy_stamp(topk_idx, n_valid, now, birth, last_access, freq, reuse_idx=None, reuse_cnt=None):
    """In place on birth/last_access/freq [B,E,S] int32: bookkeeping of the entry the next append
    writes (n_valid as it is before that append)."""
    topk_idx = _chk(topk_idx, np.int32, "topk_idx")
    n_valid = _chk(n_valid, np.int32, "n_valid")
    for a, nm in ((birth, "birth"), (last_access, "last_access"), (freq, "freq")):
        _chk(a, np.int32, nm)
    reuse_idx = _chk(reuse_idx, np.int32, "reuse_idx")
    reuse_cnt = _chk(reuse_cnt, np.int32, "reuse_cnt")
    B, E, S = birth.shape
    max_evict = 0 if reuse_idx is None else reuse_idx.shape[2]
    rc = lib().pikv_oracle_policy_stamp(B, E, S, topk_idx.shape[1], _ptr(topk_idx), _ptr(reuse_idx),
                                        _ptr(reuse_cnt), max_evict, _ptr(n_valid), int(now),
                                        _ptr(birth), _ptr(last_access), _ptr(freq))
    if rc:
        raise ValueError("pikv_oracle_policy_stamp failed: %d" % rc)


def policy_access(mass, n_valid, threshold, now, last_access, freq):
    """In place on last_access/freq: entries whose attention mass of this step (mass [B,E,S] f32)
    exceeds threshold are accessed at step `now`."""
    mass = _chk(mass, np.float32, "mass")
    n_valid = _chk(n_valid, np.int32, "n_valid")
    _chk(last_access, np.int32, "last_access")
    _chk(freq, np.int32, "freq")
    B, E, S = mass.shape
    rc = lib().pikv_oracle_policy_access(B, E, S, _ptr(n_valid), _ptr(mass), C.c_float(threshold),
                                         int(now), _ptr(last_access), _ptr(freq))
    if rc:
        raise ValueError("pikv_oracle_policy_access failed: %d" % rc)


def policy_utility(policy, n_valid, now, birth, last_access, freq, *, lam=0.0, window=0, protect=0,
                   h2o=None, out=None):
    """Utility f32 [B,E,S] of a Table 3 policy from the integer bookkeeping (entries >= n untouched)."""
    n_valid = _chk(n_valid, np.int32, "n_valid")
    for a, nm in ((birth, "birth"), (last_access, "last_access"), (freq, "freq")):
        _chk(a, np.int32, nm)
    h2o = _chk(h2o, np.float32, "h2o")
    B, E, S = birth.shape
    if out is None:
        out = np.zeros((B, E, S), np.float32)
    _chk(out, np.float32, "out")
    rc = lib().pikv_oracle_policy_utility(int(policy), B, E, S, _ptr(n_valid), int(now),
                                          C.c_float(lam), int(window), int(protect), _ptr(birth),
                                          _ptr(last_access), _ptr(freq), _ptr(h2o), _ptr(out))
    if rc:
        raise ValueError("pikv_oracle_policy_utility failed: %d" % rc)
    return out


def policy_compact(evicted_idx, evicted_cnt, n_valid, birth, last_access, freq):
    """In place on birth/last_access/freq: follow an eviction that compacted the shards
    (n_valid as it is after that eviction)."""
    evicted_idx = _chk(evicted_idx, np.int32, "evicted_idx")
    evicted_cnt = _chk(evicted_cnt, np.int32, "evicted_cnt")
    n_valid = _chk(n_valid, np.int32, "n_valid")
    for a, nm in ((birth, "birth"), (last_access, "last_access"), (freq, "freq")):
        _chk(a, np.int32, nm)
    B, E, S = birth.shape
    rc = lib().pikv_oracle_policy_compact(B, E, S, _ptr(evicted_idx), _ptr(evicted_cnt), evicted_idx.shape[2],
                                          _ptr(n_valid), _ptr(birth), _ptr(last_access), _ptr(freq))
    if rc:
        raise ValueError("pikv_oracle_policy_compact failed: %d" % rc)


def route_round_robin(rows, E, k, step):
    """Table 1 row B: idx int32 [rows,k], gates f32 [rows,k] of the score-free round-robin router."""
    idx = np.zeros((rows, k), np.int32)
    gates = np.zeros((rows, k), np.float32)
    rc = lib().pikv_oracle_route_round_robin(rows, E, k, C.c_int64(step), _ptr(idx), _ptr(gates))
    if rc:
        raise ValueError("pikv_oracle_route_round_robin failed: %d" % rc)
    return idx, gates

