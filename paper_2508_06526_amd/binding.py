"""ctypes binding of libpikv.so: same names and argument order as include/pikv.h.

Every function takes torch tensors that already live in device memory (or None for
optional pointers), passes their addresses and the current HIP stream through the C ABI,
and returns nothing but the status check.  No arithmetic happens here.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpikv.so")

F32, BF16 = 0, 1
COMBINE_LSE, COMBINE_LOCAL = 0, 1
PENALTY_LOAD_BALANCE, PENALTY_CACHE_AWARE, PENALTY_ENTROPY = 0, 1, 2
DESC_VALUE_BIAS = 1
POLICY_H2O, POLICY_SL, POLICY_LRU, POLICY_LRU_PLUS = 0, 1, 2, 3

EXPORTS = ("pikv_route", "pikv_attn_workspace_bytes", "pikv_sharded_attn", "pikv_update_utility",
           "pikv_evict", "pikv_append", "pikv_strerror", "pikv_version", "pikv_set_attn_split", "pikv_decode_step",
           "pikv_stream_read_probe",
           "pikv_set_profile_events", "pikv_router_penalty", "pikv_compress", "pikv_policy_stamp",
           "pikv_update_utility_tracked", "pikv_policy_utility", "pikv_policy_compact", "pikv_decode_step_policy", "pikv_route_round_robin",
           "pikv_sharded_attn_noalloc")


class PikvError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (where, pikv_strerror(status), status))


class PikvDesc(C.Structure):
    _fields_ = [("B", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("D", C.c_int32),
                ("E", C.c_int32), ("S", C.c_int32), ("rank", C.c_int32), ("dtype", C.c_int32),
                ("stride_h", C.c_int64), ("stride_s", C.c_int64),
                ("route_rows_per_seq", C.c_int32), ("flags", C.c_int32), ("tq", C.c_int32),
                ("reserved", C.c_int32)]

    @property
    def width(self):
        return self.rank if self.rank else self.D


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """dlopen libpikv.so (built by ``python -m paper_2508_06526_amd.build``).  Raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise OSError("libpikv.so is not built: run `python -m paper_2508_06526_amd.build` "
                      "(there is no fallback path)")
    # The binding passes torch tensors and torch streams to the library, so both must talk to
    # ONE HIP runtime: torch brings its own copy of libamdhip64, and a libpikv.so opened before
    # torch would bind to the system's copy instead - its launches on torch's streams then fail
    # (PIKV_ERR_HIP).  Importing torch first makes the already-loaded runtime the one libpikv gets.
    import torch  # noqa: F401
    lib = C.CDLL(_LIB_PATH)
    vp, i32, f32 = C.c_void_p, C.c_int32, C.c_float
    dp = C.POINTER(PikvDesc)
    lib.pikv_route.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, vp, vp, vp, vp]
    lib.pikv_route.restype = C.c_int
    lib.pikv_attn_workspace_bytes.argtypes = [dp, i32]
    lib.pikv_attn_workspace_bytes.restype = C.c_size_t
    lib.pikv_sharded_attn.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, f32,
                                      vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
    lib.pikv_sharded_attn.restype = C.c_int
    lib.pikv_sharded_attn_noalloc.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, f32,
                                              vp, vp, vp, vp, vp, vp]
    lib.pikv_sharded_attn_noalloc.restype = C.c_int
    lib.pikv_update_utility.argtypes = [dp, vp, vp, vp, vp, i32, f32, vp, vp]
    lib.pikv_update_utility.restype = C.c_int
    lib.pikv_policy_stamp.argtypes = [dp, vp, i32, vp, vp, i32, vp, i32, vp, vp, vp, vp]
    lib.pikv_policy_stamp.restype = C.c_int
    lib.pikv_update_utility_tracked.argtypes = [dp, vp, vp, vp, vp, i32, f32, vp, f32, i32, vp, vp, vp]
    lib.pikv_update_utility_tracked.restype = C.c_int
    lib.pikv_policy_utility.argtypes = [dp, i32, vp, i32, f32, i32, i32, vp, vp, vp, vp, vp, vp]
    lib.pikv_policy_utility.restype = C.c_int
    lib.pikv_policy_compact.argtypes = [dp, vp, vp, i32, vp, vp, vp, vp, vp]
    lib.pikv_policy_compact.restype = C.c_int
    lib.pikv_route_round_robin.argtypes = [i32, i32, i32, C.c_int64, vp, vp, vp]
    lib.pikv_route_round_robin.restype = C.c_int
    lib.pikv_evict.argtypes = [dp, vp, vp, i32, vp, i32, vp, vp, i32, i32, vp, vp, vp]
    lib.pikv_evict.restype = C.c_int
    lib.pikv_append.argtypes = [dp, vp, vp, vp, i32, vp, vp, i32, vp, vp, vp, vp, vp]
    lib.pikv_append.restype = C.c_int
    lib.pikv_strerror.argtypes = [C.c_int]
    lib.pikv_strerror.restype = C.c_char_p
    lib.pikv_decode_step.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, f32, f32,
                                     vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
    lib.pikv_decode_step.restype = C.c_int
    lib.pikv_decode_step_policy.argtypes = list(lib.pikv_decode_step.argtypes) + [vp, vp]
    lib.pikv_decode_step_policy.restype = C.c_int
    lib.pikv_stream_read_probe.argtypes = [vp, i32, C.c_size_t, i32, vp, vp]
    lib.pikv_stream_read_probe.restype = C.c_int
    lib.pikv_router_penalty.argtypes = [i32, vp, i32, i32, i32, vp, vp, f32, vp, vp]
    lib.pikv_router_penalty.restype = C.c_int
    lib.pikv_compress.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp]
    lib.pikv_compress.restype = C.c_int
    lib.pikv_set_profile_events.argtypes = [vp, vp]
    lib.pikv_set_profile_events.restype = None
    lib.pikv_set_attn_split.argtypes = [i32]
    lib.pikv_set_attn_split.restype = None
    lib.pikv_version.argtypes = []
    lib.pikv_version.restype = C.c_int
    _lib = lib
    return lib


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError("storage dtype must be float32 or bfloat16, got %s" % t.dtype)


def _p(t):
    """Device address of a tensor (None -> NULL)."""
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("libpikv takes device memory only")
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _check(status, where):
    if status != 0:
        raise PikvError(status, where)


def make_desc(B, Hq, Hkv, D, E, S, rank=0, dtype=BF16, stride_h=None, stride_s=None,
              route_rows_per_seq=1, flags=0, tq=1) -> PikvDesc:
    w = rank if rank else D
    if stride_s is None:
        stride_s = w
    if stride_h is None:
        stride_h = S * stride_s
    return PikvDesc(B, Hq, Hkv, D, E, S, rank, dtype, stride_h, stride_s, route_rows_per_seq, flags, tq, 0)


def shard_table(shards, device=None):
    """Device array of B*E shard base addresses (entry b*E+e).

    ``shards`` is a tensor [B,E,Hkv,S,w] (one allocation) or a flat list of B*E tensors.
    """
    import torch
    if isinstance(shards, torch.Tensor):
        B, E = shards.shape[:2]
        step = shards.stride(1) * shards.element_size()
        assert shards.stride(0) == E * shards.stride(1)
        ptrs = [shards.data_ptr() + i * step for i in range(B * E)]
        device = shards.device
    else:
        ptrs = [s.data_ptr() for s in shards]
        device = shards[0].device
    return torch.tensor(ptrs, dtype=torch.int64, device=device)


def pikv_strerror(status: int) -> str:
    return load_library().pikv_strerror(int(status)).decode()


def pikv_version() -> int:
    return load_library().pikv_version()


def pikv_set_attn_split(nsplit: int) -> None:
    load_library().pikv_set_attn_split(int(nsplit))


def pikv_set_profile_events(start, stop) -> None:
    """start/stop: torch.cuda.Event (timing enabled, already recorded once so that the HIP
    event exists) or None/None to switch the hook off."""
    h = lambda ev: None if ev is None else C.c_void_p(ev.cuda_event)
    load_library().pikv_set_profile_events(h(start), h(stop))


def pikv_route(x, W_r, bias, rows, d_r, E, k, topk_idx, gates, probs=None, stream=None):
    st = load_library().pikv_route(_p(x), _p(W_r), _p(bias), rows, d_r, E, k, _dtype_code(x),
                                   _p(topk_idx), _p(gates), _p(probs), _stream(stream))
    _check(st, "pikv_route")


def pikv_attn_workspace_bytes(desc: PikvDesc, k: int) -> int:
    return int(load_library().pikv_attn_workspace_bytes(C.byref(desc), k))


def pikv_sharded_attn(desc, q, K_shards, V_shards, U_K, U_V, n_valid, topk_idx, gates, k, combine,
                      scale, y, row_max, row_norm, scores, slot_coef, workspace, stream=None):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = load_library().pikv_sharded_attn(
        C.byref(desc), _p(q), _p(K_shards), _p(V_shards), _p(U_K), _p(U_V), _p(n_valid),
        _p(topk_idx), _p(gates), k, combine, float(scale), _p(y), _p(row_max), _p(row_norm),
        _p(scores), _p(slot_coef), _p(workspace), ws_bytes, _stream(stream))
    _check(st, "pikv_sharded_attn")


NOALLOC_SCRATCH_BYTES = 4 << 20


def pikv_sharded_attn_noalloc(desc, q, K_shards, V_shards, U_K, U_V, n_valid, topk_idx, gates, k, combine,
                              scale, y, row_max, row_norm, scores, slot_coef, stream=None):
    st = load_library().pikv_sharded_attn_noalloc(
        C.byref(desc), _p(q), _p(K_shards), _p(V_shards), _p(U_K), _p(U_V), _p(n_valid),
        _p(topk_idx), _p(gates), k, combine, float(scale), _p(y), _p(row_max), _p(row_norm),
        _p(scores), _p(slot_coef), _stream(stream))
    _check(st, "pikv_sharded_attn_noalloc")


def pikv_update_utility(desc, scores, slot_coef, n_valid, topk_idx, k, decay, utility, stream=None):
    st = load_library().pikv_update_utility(C.byref(desc), _p(scores), _p(slot_coef), _p(n_valid),
                                            _p(topk_idx), k, float(decay), _p(utility),
                                            _stream(stream))
    _check(st, "pikv_update_utility")


def pikv_evict(desc, utility, n_valid, capacity, sel_idx, sel_k, evicted_idx, evicted_cnt,
               max_evict, compact, K_shards, V_shards, stream=None):
    st = load_library().pikv_evict(C.byref(desc), _p(utility), _p(n_valid), capacity, _p(sel_idx),
                                   sel_k, _p(evicted_idx), _p(evicted_cnt), max_evict,
                                   1 if compact else 0, _p(K_shards), _p(V_shards), _stream(stream))
    _check(st, "pikv_evict")


def pikv_append(desc, K_new, V_new, topk_idx, k, reuse_idx, reuse_cnt, max_evict, K_shards,
                V_shards, utility, n_valid, stream=None):
    st = load_library().pikv_append(C.byref(desc), _p(K_new), _p(V_new), _p(topk_idx), k,
                                    _p(reuse_idx), _p(reuse_cnt), max_evict, _p(K_shards),
                                    _p(V_shards), _p(utility), _p(n_valid), _stream(stream))
    _check(st, "pikv_append")


def pikv_decode_step(desc, q, W_r, bias, K_new, V_new, K_shards, V_shards, U_K, U_V, n_valid, utility,
                     k, combine, scale, decay, topk_idx, gates, evicted_idx, evicted_cnt, y, row_max,
                     row_norm, scores, slot_coef, workspace, stream=None):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = load_library().pikv_decode_step(
        C.byref(desc), _p(q), _p(W_r), _p(bias), _p(K_new), _p(V_new), _p(K_shards), _p(V_shards),
        _p(U_K), _p(U_V), _p(n_valid), _p(utility), k, combine, float(scale), float(decay),
        _p(topk_idx), _p(gates), _p(evicted_idx), _p(evicted_cnt), _p(y), _p(row_max), _p(row_norm),
        _p(scores), _p(slot_coef), _p(workspace), ws_bytes, _stream(stream))
    _check(st, "pikv_decode_step")


def pikv_stream_read_probe(bufs, n, bytes_each, parts, out, stream=None):
    st = load_library().pikv_stream_read_probe(_p(bufs), n, bytes_each, parts, _p(out), _stream(stream))
    _check(st, "pikv_stream_read_probe")


def pikv_router_penalty(mode, topk_idx, rows, k, E, load, miss, coef, bias, stream=None):
    st = load_library().pikv_router_penalty(mode, _p(topk_idx), rows, k, E, _p(load), _p(miss),
                                            float(coef), _p(bias), _stream(stream))
    _check(st, "pikv_router_penalty")


def pikv_compress(desc, K_full, Wenc_K, K_codes, V_full=None, Wenc_V=None, V_codes=None, stream=None):
    st = load_library().pikv_compress(C.byref(desc), _p(K_full), _p(Wenc_K), _p(K_codes), _p(V_full),
                                      _p(Wenc_V), _p(V_codes), _stream(stream))
    _check(st, "pikv_compress")


def pikv_policy_stamp(desc, topk_idx, k, reuse_idx, reuse_cnt, max_evict, n_valid, now, birth,
                      last_access, freq, stream=None):
    st = load_library().pikv_policy_stamp(C.byref(desc), _p(topk_idx), k, _p(reuse_idx), _p(reuse_cnt),
                                          max_evict, _p(n_valid), int(now), _p(birth), _p(last_access),
                                          _p(freq), _stream(stream))
    _check(st, "pikv_policy_stamp")


def pikv_update_utility_tracked(desc, scores, slot_coef, n_valid, topk_idx, k, decay, utility, threshold,
                                now, last_access, freq, stream=None):
    st = load_library().pikv_update_utility_tracked(C.byref(desc), _p(scores), _p(slot_coef), _p(n_valid),
                                                    _p(topk_idx), k, float(decay), _p(utility),
                                                    float(threshold), int(now), _p(last_access), _p(freq),
                                                    _stream(stream))
    _check(st, "pikv_update_utility_tracked")


def pikv_policy_utility(desc, policy, n_valid, now, lam, window, protect, birth, last_access, freq, h2o,
                        out, stream=None):
    st = load_library().pikv_policy_utility(C.byref(desc), int(policy), _p(n_valid), int(now), float(lam),
                                            int(window), int(protect), _p(birth), _p(last_access),
                                            _p(freq), _p(h2o), _p(out), _stream(stream))
    _check(st, "pikv_policy_utility")


def pikv_policy_compact(desc, evicted_idx, evicted_cnt, max_evict, n_valid, birth, last_access, freq,
                        stream=None):
    st = load_library().pikv_policy_compact(C.byref(desc), _p(evicted_idx), _p(evicted_cnt), max_evict,
                                            _p(n_valid), _p(birth), _p(last_access), _p(freq), _stream(stream))
    _check(st, "pikv_policy_compact")


class PikvPolicyArgs(C.Structure):
    _fields_ = [("policy", C.c_int32), ("now", C.c_int32), ("lam", C.c_float), ("window", C.c_int32),
                ("protect", C.c_int32), ("threshold", C.c_float), ("birth", C.c_void_p),
                ("last_access", C.c_void_p), ("freq", C.c_void_p)]


def make_policy_args(policy, now, lam=0.0, window=0, protect=0, threshold=0.0, birth=None, last_access=None,
                     freq=None):
    a = PikvPolicyArgs()
    a.policy, a.now, a.lam, a.window, a.protect, a.threshold = int(policy), int(now), float(lam), int(window), \
        int(protect), float(threshold)
    for name, t in (("birth", birth), ("last_access", last_access), ("freq", freq)):
        ptr = _p(t)
        setattr(a, name, None if ptr is None else ptr.value)
    return a


class PikvRouterFeedback(C.Structure):
    _fields_ = [("mode", C.c_int32), ("coef", C.c_float), ("load", C.c_void_p), ("miss", C.c_void_p),
                ("bias", C.c_void_p)]


def make_router_feedback(mode, coef, load, bias, miss=None):
    f = PikvRouterFeedback()
    f.mode, f.coef = int(mode), float(coef)
    for name, t in (("load", load), ("miss", miss), ("bias", bias)):
        ptr = _p(t)
        setattr(f, name, None if ptr is None else ptr.value)
    return f


def pikv_decode_step_policy(desc, q, W_r, bias, K_new, V_new, K_shards, V_shards, U_K, U_V, n_valid, utility, k,
                            combine, scale, decay, topk_idx, gates, evicted_idx, evicted_cnt, y, row_max,
                            row_norm, scores, slot_coef, workspace, policy_args, feedback=None, stream=None):
    st = load_library().pikv_decode_step_policy(
        C.byref(desc), _p(q), _p(W_r), _p(bias), _p(K_new), _p(V_new), _p(K_shards), _p(V_shards), _p(U_K),
        _p(U_V), _p(n_valid), _p(utility), k, combine, float(scale), float(decay), _p(topk_idx), _p(gates),
        _p(evicted_idx), _p(evicted_cnt), _p(y), _p(row_max), _p(row_norm), _p(scores), _p(slot_coef),
        _p(workspace), workspace.numel() * workspace.element_size(), _stream(stream),
        None if policy_args is None else C.cast(C.pointer(policy_args), C.c_void_p),
        None if feedback is None else C.cast(C.pointer(feedback), C.c_void_p))
    _check(st, "pikv_decode_step_policy")


def pikv_route_round_robin(rows, E, k, step, topk_idx, gates, stream=None):
    st = load_library().pikv_route_round_robin(rows, E, k, int(step), _p(topk_idx), _p(gates), _stream(stream))
    _check(st, "pikv_route_round_robin")

