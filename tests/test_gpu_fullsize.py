"""Parity at the full workload sizes, in the launch configuration bench.py times
(`pikv_decode_step` on device-generated layers, the library's own split policy).

Exact things are checked for every row / shard (expert indices, evicted slots on the GPU's own
pre-step utility bits, inserted rows, entry counts); attention outputs and utilities are
checked against the oracle for whole sequences (all heads, all selected entries), for every
sequence of every workload (the oracle and the host copies of the shards finish in seconds).
"""
import numpy as np
import pytest

import workloads as wl
from oracle import pikv_oracle as orc

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():  # pragma: no cover
    pytest.skip("no GPU", allow_module_level=True)

import bench  # noqa: E402
import paper_2508_06526_amd as pk  # noqa: E402
from gpu_harness import DEV, assert_utility_close, dev_storage, t2n, y_tolerance_ok  # noqa: E402

FULL = {
    # name: (sequences checked against the oracle, decay)
    "c2_bf16_decode": (list(range(8)), 1.0),
    "c3_long_context": ([0], 1.0),
    "c4_streaming": (list(range(32)), 0.9),
    "c5_compressed": (list(range(16)), 1.0),
    # "next" row: 4 draft queries per sequence share the selected shards (group of 16 query rows)
    "c3_long_context_tq4": ([0], 1.0),
    # wider tiles in the tokens' natural layout (desc.tq): 32 and 64 query rows per kv head
    "c3_long_context_tq8": ([0], 1.0),
    "c3_kv4_tq16": ([0], 1.0),
}


def redraw_for_margin(geo, q_host, W_host, bias_host, k, seed0=77_000):
    """Host-side margin filter (oracle logits in fp64), see gpu_harness.ensure_route_margin."""
    q = q_host.copy()
    for attempt in range(50):
        x = np.ascontiguousarray(wl.routing_rows(geo, q))
        _, _, _, logits = orc.route(x, W_host, k, bias=bias_host, dtype=geo.dtype, want_logits=True)
        srt = -np.sort(-logits, axis=1)
        bad = np.nonzero(np.abs(np.diff(srt[:, :k + 1], axis=1)).min(axis=1) < 1e-3)[0]
        if bad.size == 0:
            return q
        fresh = wl.draw_queries(geo, seed0 + attempt).reshape(geo.route_rows, -1)
        q = q.reshape(geo.route_rows, -1).copy()
        q[bad] = fresh[bad]
        q = np.ascontiguousarray(q.reshape(geo.B, geo.Hq, geo.D))
    raise AssertionError("routing margin not reached")


@pytest.mark.parametrize("name", sorted(FULL))
def test_full_size_step_matches_oracle(name):
    seqs, decay = FULL[name]
    geo = wl.CONFIGS[name]
    dev = torch.device(DEV)
    raw = wl.make_device_layers(geo, 1, 123, dev, **bench.RECIPE[name])
    bench.DECAY.setdefault(name, decay)
    shared = bench.make_shared(pk, torch, geo, dev)
    shared["fused"] = True
    L = bench.Layer(pk, torch, geo, raw[0], shared)
    t = L.t
    if name != "c4_streaming":          # give every layer distinct, positive starting utilities
        t["utility"].exponential_(1.0).div_(geo.S)
    # routing margin, so that fp32 summation order cannot change the selection
    W_host = wl.to_host(t["W_r"], geo.dtype)
    bias_host = None if t["bias"] is None else t["bias"].cpu().numpy()
    q_host = redraw_for_margin(geo, wl.to_host(t["q"], geo.dtype), W_host, bias_host, geo.k)
    t["q"].copy_(dev_storage(q_host, geo.dtype))
    u_before, n_before = t2n(t["utility"]), t2n(t["n_valid"])

    L.step()                              # pikv_decode_step, as in the benchmark
    torch.cuda.synchronize()

    # --- exact: routing for every row
    x = np.ascontiguousarray(wl.routing_rows(geo, q_host))      # q_host is in the caller's layout
    idx, gates, _ = orc.route(x, W_host, geo.k, bias=bias_host, dtype=geo.dtype)
    np.testing.assert_array_equal(t2n(shared["topk"]), idx)
    np.testing.assert_allclose(t2n(shared["gates"]), gates, rtol=2e-5, atol=1e-7)
    # --- exact: eviction of every selected full shard, on the GPU's own pre-step bits
    mask = np.zeros((geo.B, geo.E), np.int32)
    for b in range(geo.B):
        mask[b, idx[b]] = 1
    u_ref, n_ref = u_before.copy(), n_before.copy()
    ridx, rcnt = orc.evict(u_ref, n_ref, geo.S - 1, shard_mask=mask, max_evict=1)
    ecnt, eidx = t2n(shared["ecnt"]), t2n(shared["eidx"])
    np.testing.assert_array_equal(ecnt, rcnt)
    np.testing.assert_array_equal(eidx[rcnt == 1], ridx[rcnt == 1])
    assert (rcnt[mask == 1] == 1).all()                      # every shard of these workloads is full
    np.testing.assert_array_equal(t2n(t["n_valid"]), n_before)
    # --- exact: the new rows sit in the freed slots (every selected shard)
    kn, vn = wl.to_host(shared["K_new"], geo.dtype), wl.to_host(shared["V_new"], geo.dtype)
    for b in range(geo.B):
        for e in idx[b]:
            slot = int(ridx[b, e, 0])
            np.testing.assert_array_equal(wl.to_host(t["K"][b, e, :, slot], geo.dtype), kn[b])
            np.testing.assert_array_equal(wl.to_host(t["V"][b, e, :, slot], geo.dtype), vn[b])

    # --- tolerance: attention output and utilities of whole sequences via the oracle
    y_gpu, u_gpu = t2n(shared["y"]), t2n(t["utility"])
    q_orc = q_host
    if geo.token_major:       # the oracle takes the same rows in kv-head-first order
        perm = wl.token_major_rows(geo.Hq, geo.Hkv, geo.tq)
        q_orc = np.ascontiguousarray(q_host[:, perm])
        y_gpu = np.ascontiguousarray(y_gpu[:, perm])
    dummy = np.zeros((1,), np.float32 if geo.dtype == "f32" else np.uint16)
    UK = None if t["U_K"] is None else wl.to_host(t["U_K"], geo.dtype)
    UV = None if t["U_V"] is None else wl.to_host(t["U_V"], geo.dtype)
    for b in seqs:
        Ks, Vs = [dummy] * geo.E, [dummy] * geo.E
        for e in idx[b]:
            Ks[e] = wl.to_host(t["K"][b, e], geo.dtype)       # post-insert contents
            Vs[e] = wl.to_host(t["V"][b, e], geo.dtype)
        u_seq = u_before[b:b + 1].copy()
        for e in idx[b]:
            u_seq[0, e, int(ridx[b, e, 0])] = 0.0             # the inserted entry starts at 0
        out = orc.attend(np.ascontiguousarray(q_orc[b:b + 1]), Ks, Vs,
                         np.ascontiguousarray(n_before[b:b + 1]), np.ascontiguousarray(idx[b:b + 1]),
                         np.ascontiguousarray(gates[b:b + 1]), Hkv=geo.Hkv, E=geo.E, S=geo.S,
                         dtype=geo.dtype, rank=geo.rank, U_K=UK, U_V=UV, utility=u_seq, decay=decay)
        ok, emax, l2 = y_tolerance_ok(y_gpu[b:b + 1], out["y"], geo.dtype)
        assert ok, "%s seq %d: max abs %.3e rel L2 %.3e" % (name, b, emax, l2)
        assert_utility_close(u_gpu[b], u_seq[0])
    # property at any size: attention mass added to each sequence equals the number of query heads
    u_after = u_gpu.astype(np.float64)
    base = u_before.astype(np.float64)
    for b in range(geo.B):
        for e in idx[b]:
            base[b, e, int(ridx[b, e, 0])] = 0.0
    for b in range(geo.B):
        sel = idx[b]
        added = (u_after[b, sel] - decay * base[b, sel]).sum()
        np.testing.assert_allclose(added, geo.Hq, rtol=2e-4)
        rest = [e for e in range(geo.E) if e not in set(sel.tolist())]
        np.testing.assert_array_equal(u_gpu[b, rest], u_before[b, rest])
