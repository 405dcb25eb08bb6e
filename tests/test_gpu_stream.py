"""The streaming workload as a chain: 256 consecutive decode steps (route -> evict the
minimum-utility entry of every selected full shard -> insert -> attend -> utility with decay
0.9) through pikv_decode_step, at the streaming configuration's shard shape (32 heads, D = 128,
E = 8 shards of 2048, k = 2) with enough streams for more than one round of attention blocks -
the launch configuration the benchmark times - compared step by step with the oracle under the
protocol of stream_protocol.py."""
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
from stream_protocol import reconcile_eviction  # noqa: E402

STEPS = 256


def margin_queries(geo, W_host, seed):
    """A query batch whose routing decision no fp32 summation order can change."""
    q = wl.draw_queries(geo, seed)
    for attempt in range(50):
        x = np.ascontiguousarray(q.reshape(geo.route_rows, geo.d_r))
        _, _, _, logits = orc.route(x, W_host, geo.k, dtype=geo.dtype, want_logits=True)
        srt = -np.sort(-logits, axis=1)
        bad = np.nonzero(np.abs(np.diff(srt[:, :geo.k + 1], axis=1)).min(axis=1) < 1e-3)[0]
        if bad.size == 0:
            return q
        fresh = wl.draw_queries(geo, seed + 1000 * (attempt + 1)).reshape(geo.route_rows, geo.d_r)
        x = x.copy()
        x[bad] = fresh[bad]
        q = np.ascontiguousarray(x.reshape(geo.B, geo.Hq, geo.D))
    raise AssertionError("routing margin not reached")


def test_streaming_chain_of_256_steps_matches_the_oracle():
    geo = wl.Geometry(B=20, Hq=32, Hkv=32, D=128, E=8, S=2048, k=2, dtype="bf16", name="c4_chain")
    dev = torch.device(DEV)
    raw = wl.make_device_layers(geo, 1, 321, dev, utility0="exp")
    shared = bench.make_shared(pk, torch, geo, dev)
    shared["fused"] = True
    L = bench.Layer(pk, torch, geo, raw[0], shared)
    L.decay = 0.9
    t = L.t
    plan_blocks = geo.B * geo.Hq * geo.k           # one block per (stream, head, shard) at least
    assert plan_blocks > 1024, "the chain is meant to need more than one round of attention blocks"

    # the oracle's free-running state
    W_host = wl.to_host(t["W_r"], geo.dtype)
    Ks = [wl.to_host(t["K"][b, e], geo.dtype) for b in range(geo.B) for e in range(geo.E)]
    Vs = [wl.to_host(t["V"][b, e], geo.dtype) for b in range(geo.B) for e in range(geo.E)]
    u_ref, n_ref = t2n(t["utility"]), t2n(t["n_valid"])
    adopted_total, y_worst, first_adoption = 0, 0.0, None
    for step in range(STEPS):
        q = margin_queries(geo, W_host, 40_000 + step)
        kn, vn = wl.draw_new_kv(geo, 50_000 + step)
        t["q"].copy_(dev_storage(q, geo.dtype))
        shared["K_new"].copy_(dev_storage(kn, geo.dtype))
        shared["V_new"].copy_(dev_storage(vn, geo.dtype))
        u_before, n_before = t2n(t["utility"]), t2n(t["n_valid"])
        L.step()                                    # pikv_decode_step, decay 0.9
        torch.cuda.synchronize()

        x = np.ascontiguousarray(q.reshape(geo.route_rows, geo.d_r))
        idx, gates, _ = orc.route(x, W_host, geo.k, dtype=geo.dtype)
        np.testing.assert_array_equal(t2n(shared["topk"]), idx, err_msg="step %d" % step)
        mask = np.zeros((geo.B, geo.E), np.int32)
        for b in range(geo.B):
            mask[b, idx[b]] = 1
        ridx, rcnt, adopted = reconcile_eviction(u_ref, n_ref, geo.S, mask, t2n(shared["eidx"]),
                                                 t2n(shared["ecnt"]), u_before, n_before, step)
        if adopted and first_adoption is None:
            first_adoption = step
        adopted_total += adopted
        assert (rcnt[mask == 1] == 1).all()         # every shard of this workload stays full
        orc.append(kn, vn, idx, Ks, Vs, u_ref, n_ref, dtype=geo.dtype, reuse_idx=ridx, reuse_cnt=rcnt)
        out = orc.attend(q, Ks, Vs, n_ref, idx, gates, Hkv=geo.Hkv, E=geo.E, S=geo.S, dtype=geo.dtype,
                         utility=u_ref, decay=0.9)
        ok, emax, l2 = y_tolerance_ok(t2n(shared["y"]), out["y"], geo.dtype)
        assert ok, "step %d: max abs %.3e rel L2 %.3e" % (step, emax, l2)
        y_worst = max(y_worst, l2)
        assert_utility_close(t2n(t["utility"]), u_ref)          # rel 1e-4 after `step + 1` decayed updates
        np.testing.assert_array_equal(t2n(t["n_valid"]), n_ref)
    # the caches hold the same entries in the same slots at the end (a sample of shards)
    for b, e in ((0, 0), (7, 3), (geo.B - 1, geo.E - 1)):
        np.testing.assert_array_equal(wl.to_host(t["K"][b, e], geo.dtype), Ks[b * geo.E + e])
        np.testing.assert_array_equal(wl.to_host(t["V"][b, e], geo.dtype), Vs[b * geo.E + e])
    print("chain of %d steps: %d near-tie evictions adopted (first at step %s), worst rel L2 of y %.2e"
          % (STEPS, adopted_total, first_adoption, y_worst))
