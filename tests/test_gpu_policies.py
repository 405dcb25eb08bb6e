"""Scheduling policies of Table 3 (SL, LRU, LRU+, recent-entry protection): HIP path vs oracle.

Integer bookkeeping (insertion stamp, last-access stamp, access count), the policy utilities
and the evicted slots are compared bit for bit.  The one place floating point decides an
integer - "attention mass above the threshold" - is kept away from the decision boundary: the
threshold of a step is put in the middle of a wide gap of the oracle's masses.
"""
import numpy as np
import pytest

import workloads as wl
from oracle import pikv_oracle as orc

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():  # pragma: no cover
    pytest.skip("no GPU", allow_module_level=True)

import paper_2508_06526_amd as pk  # noqa: E402
from gpu_harness import (DEV, DeviceCase, assert_utility_close, dev_storage, ensure_route_margin,  # noqa: E402
                         t2n)

POLICIES = {"h2o": (pk.POLICY_H2O, orc.POLICY_H2O), "sl": (pk.POLICY_SL, orc.POLICY_SL),
            "lru": (pk.POLICY_LRU, orc.POLICY_LRU), "lru_plus": (pk.POLICY_LRU_PLUS, orc.POLICY_LRU_PLUS)}


def to_dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def random_state(rng, B, E, S, now):
    birth = rng.integers(0, now + 1, size=(B, E, S)).astype(np.int32)
    last = np.maximum(birth, rng.integers(0, now + 1, size=(B, E, S))).astype(np.int32)
    freq = rng.integers(0, 3000, size=(B, E, S)).astype(np.int32)
    return birth, last, freq


@pytest.mark.parametrize("name", sorted(POLICIES))
@pytest.mark.parametrize("protect", [0, 40])
def test_policy_utility_matches_oracle_bit_exact(name, protect):
    g = wl.Geometry(B=3, Hq=2, Hkv=2, D=16, E=5, S=700, k=2, dtype="bf16")
    rng = np.random.default_rng(11)
    now = 5000
    birth, last, freq = random_state(rng, g.B, g.E, g.S, now)
    n = rng.integers(0, g.S + 1, size=(g.B, g.E)).astype(np.int32)
    n[0, 0], n[0, 1] = g.S, 0
    h2o = rng.random((g.B, g.E, g.S)).astype(np.float32)
    lam = float(np.float32(0.37))                     # products that need rounding
    ref = orc.policy_utility(POLICIES[name][1], n, now, birth, last, freq, lam=lam, window=900,
                             protect=protect, h2o=h2o, out=np.full((g.B, g.E, g.S), -7.0, np.float32))
    desc = pk.make_desc(g.B, g.Hq, g.Hkv, g.D, g.E, g.S, dtype=1)
    out = torch.full((g.B, g.E, g.S), -7.0, device=DEV)
    pk.pikv_policy_utility(desc, POLICIES[name][0], to_dev(n), now, lam, 900, protect, to_dev(birth),
                           to_dev(last), to_dev(freq), to_dev(h2o), out)
    got = t2n(out)
    np.testing.assert_array_equal(got.view(np.uint32), ref.view(np.uint32))   # bits, dead slots untouched
    # and the decision they feed: the same evicted slots
    cap = g.S // 2
    ridx, rcnt = orc.evict(ref.copy(), n.copy(), cap)
    eidx = torch.full((g.B, g.E, g.S), -1, device=DEV, dtype=torch.int32)
    ecnt = torch.zeros((g.B, g.E), device=DEV, dtype=torch.int32)
    nd = to_dev(n)
    pk.pikv_evict(desc, out, nd, cap, None, 0, eidx, ecnt, g.S, False, None, None)
    np.testing.assert_array_equal(t2n(ecnt), rcnt)
    e_host = t2n(eidx)
    for b in range(g.B):
        for e in range(g.E):
            np.testing.assert_array_equal(e_host[b, e, :rcnt[b, e]], ridx[b, e, :rcnt[b, e]])


def test_policy_stamp_matches_oracle():
    g = wl.Geometry(B=4, Hq=2, Hkv=2, D=16, E=6, S=20, k=3, dtype="bf16")
    rng = np.random.default_rng(12)
    birth, last, freq = random_state(rng, g.B, g.E, g.S, 100)
    n = rng.integers(0, g.S, size=(g.B, g.E)).astype(np.int32)      # never full: the oracle rejects that
    topk = np.stack([rng.permutation(g.E)[:g.k] for _ in range(g.B)]).astype(np.int32)
    reuse_idx = rng.integers(0, g.S, size=(g.B, g.E, 2)).astype(np.int32)
    reuse_cnt = rng.integers(0, 2, size=(g.B, g.E)).astype(np.int32)
    desc = pk.make_desc(g.B, g.Hq, g.Hkv, g.D, g.E, g.S, dtype=1)
    d = [to_dev(a) for a in (birth, last, freq)]
    pk.pikv_policy_stamp(desc, to_dev(topk), g.k, to_dev(reuse_idx), to_dev(reuse_cnt), 2, to_dev(n), 123,
                         d[0], d[1], d[2])
    orc.policy_stamp(topk, n, 123, birth, last, freq, reuse_idx, reuse_cnt)
    for got, ref in zip(d, (birth, last, freq)):
        np.testing.assert_array_equal(t2n(got), ref)
    assert (birth == 123).sum() == g.B * g.k
    # without a reuse list; a full shard is skipped (its insert is dropped too)
    n[0, topk[0, 0]] = g.S
    before = [t2n(x).copy() for x in d]
    pk.pikv_policy_stamp(desc, to_dev(topk), g.k, None, None, 0, to_dev(n), 124, d[0], d[1], d[2])
    now_b = t2n(d[0])
    assert (now_b[0, topk[0, 0]] == before[0][0, topk[0, 0]]).all()
    assert (now_b == 124).sum() == g.B * g.k - 1
    for b in range(g.B):
        for e in topk[b]:
            if n[b, e] < g.S:
                assert now_b[b, e, n[b, e]] == 124


def threshold_in_a_gap(mass, n, quantile):
    """A threshold near the given quantile of the live masses with a wide relative margin to
    every mass, so that fp32 summation order cannot move an entry across it."""
    live = np.concatenate([mass[b, e, :n[b, e]] for b in range(n.shape[0]) for e in range(n.shape[1])])
    live = np.unique(live[live > 0])
    assert live.size > 8
    c = int(quantile * (live.size - 1))
    lo, hi = max(0, c - 6), min(live.size - 1, c + 6)
    ratios = live[lo + 1:hi + 1] / live[lo:hi]
    j = lo + int(np.argmax(ratios))
    assert ratios.max() > 1.0 + 1e-3, "no gap wide enough near the quantile"
    return float(np.float32(np.sqrt(float(live[j]) * float(live[j + 1]))))


@pytest.mark.parametrize("spec", [
    dict(B=3, Hq=8, Hkv=2, D=64, E=4, S=300, k=2, dtype="bf16"),
    dict(B=2, Hq=4, Hkv=4, D=128, E=6, S=130, k=3, dtype="bf16", rank=32),
    dict(B=1, Hq=4, Hkv=4, D=64, E=4, S=256, k=2, dtype="f32", per_head_routing=True),
], ids=["gqa4", "rank32", "c1_per_head"])
@pytest.mark.parametrize("with_utility", [True, False], ids=["u", "no_u"])
def test_tracked_utility_update_matches_oracle(spec, with_utility):
    g = wl.Geometry(**spec)
    case = wl.make_host_case(g, seed=51, n_valid="ragged", utility0="exp",
                             w_sigma=1.0 if g.dtype == "f32" else 0.02)
    ensure_route_margin(case, g.k)
    dc = DeviceCase(case)
    dc.route()
    dc.attend()
    idx, gates = t2n(dc.topk), t2n(dc.gates)
    # the oracle's attention mass of this step: a utility update from zero with no history
    mass = np.zeros((g.B, g.E, g.S), np.float32)
    orc.attend(case.q, case.K_shards, case.V_shards, case.n_valid, idx, gates, Hkv=g.Hkv, E=g.E, S=g.S,
               dtype=g.dtype, rank=g.rank, U_K=case.U_K, U_V=case.U_V, utility=mass, decay=0.0)
    thr = threshold_in_a_gap(mass, case.n_valid, 0.6)
    rng = np.random.default_rng(13)
    birth, last, freq = random_state(rng, g.B, g.E, g.S, 50)
    d_last, d_freq = to_dev(last), to_dev(freq)
    u_ref = case.utility.copy()
    pk.pikv_update_utility_tracked(dc.desc, dc.scores, dc.slot_coef, dc.n_valid, dc.topk, g.k, 0.8,
                                   dc.utility if with_utility else None, thr, 77, d_last, d_freq)
    orc.policy_access(mass, case.n_valid, thr, 77, last, freq)
    np.testing.assert_array_equal(t2n(d_last), last)
    np.testing.assert_array_equal(t2n(d_freq), freq)
    assert 0 < (last == 77).sum() < last.size
    if with_utility:
        visited = np.zeros((g.B, g.E), bool)
        for r in range(idx.shape[0]):
            visited[r // g.Hq if g.per_head_routing else r, idx[r]] = True
        u_ref = np.where(visited[:, :, None] & (np.arange(g.S) < case.n_valid[:, :, None]),
                         np.float32(0.8) * u_ref + mass, u_ref)
        assert_utility_close(t2n(dc.utility), u_ref)
    else:
        np.testing.assert_array_equal(t2n(dc.utility), case.utility)


@pytest.mark.parametrize("name", ["lru", "lru_plus", "sl"])
def test_streaming_with_a_bookkeeping_policy(name):
    """route -> policy utility -> evict 1 from every selected full shard -> stamp -> append ->
    attend -> tracked update, for several steps; both sides free running.  Selections, evicted
    slots and all three integer arrays stay equal."""
    g = wl.Geometry(B=3, Hq=4, Hkv=2, D=64, E=4, S=48, k=2, dtype="bf16")
    case = wl.make_host_case(g, seed=61, utility0="exp")
    case.n_valid[:, 1] = g.S - 2
    dc = DeviceCase(case)
    ref = case.clone()
    rng = np.random.default_rng(14)
    birth, last, freq = random_state(rng, g.B, g.E, g.S, 30)
    d_birth, d_last, d_freq = to_dev(birth), to_dev(last), to_dev(freq)
    u_pol = torch.zeros((g.B, g.E, g.S), device=DEV)
    eidx = torch.full((g.B, g.E, 1), -1, device=DEV, dtype=torch.int32)
    ecnt = torch.zeros((g.B, g.E), device=DEV, dtype=torch.int32)
    gp, op = POLICIES[name]
    lam, window = 2.5, 20
    evicted_any = 0
    for step in range(10):
        now = 31 + step
        probe = case.clone()
        probe.q = wl.draw_queries(g, 600 + step)
        ensure_route_margin(probe, g.k)
        qn = probe.q
        kn, vn = wl.draw_new_kv(g, 650 + step)
        # ---- oracle
        x = np.ascontiguousarray(qn.reshape(g.route_rows, g.d_r))
        idx, gates, _ = orc.route(x, ref.W_r, g.k, dtype=g.dtype)
        mask = np.zeros((g.B, g.E), np.int32)
        for b in range(g.B):
            mask[b, idx[b]] = 1
        u_o = orc.policy_utility(op, ref.n_valid, now, birth, last, freq, lam=lam, window=window)
        ridx, rcnt = orc.evict(u_o, ref.n_valid, g.S - 1, shard_mask=mask, max_evict=1)
        orc.policy_stamp(idx, ref.n_valid, now, birth, last, freq, ridx, rcnt)
        orc.append(kn, vn, idx, ref.K_shards, ref.V_shards, ref.utility, ref.n_valid, dtype=g.dtype,
                   reuse_idx=ridx, reuse_cnt=rcnt)
        ref.q = qn
        mass = np.zeros((g.B, g.E, g.S), np.float32)
        orc.attend(ref.q, ref.K_shards, ref.V_shards, ref.n_valid, idx, gates, Hkv=g.Hkv, E=g.E, S=g.S,
                   dtype=g.dtype, utility=mass, decay=0.0)
        thr = threshold_in_a_gap(mass, ref.n_valid, 0.5)
        orc.policy_access(mass, ref.n_valid, thr, now, last, freq)
        # ---- GPU
        dc.q.copy_(dev_storage(qn, g.dtype))
        dc.route()
        pk.pikv_policy_utility(dc.desc, gp, dc.n_valid, now, lam, window, 0, d_birth, d_last, d_freq, None,
                               u_pol)
        pk.pikv_evict(dc.desc, u_pol, dc.n_valid, g.S - 1, dc.topk, g.k, eidx, ecnt, 1, False, None, None)
        pk.pikv_policy_stamp(dc.desc, dc.topk, g.k, eidx, ecnt, 1, dc.n_valid, now, d_birth, d_last, d_freq)
        pk.pikv_append(dc.desc, dev_storage(kn, g.dtype), dev_storage(vn, g.dtype), dc.topk, g.k, eidx, ecnt,
                       1, dc.K_tab, dc.V_tab, dc.utility, dc.n_valid)
        dc.attend()
        pk.pikv_update_utility_tracked(dc.desc, dc.scores, dc.slot_coef, dc.n_valid, dc.topk, g.k, 1.0, None,
                                       thr, now, d_last, d_freq)
        # ---- compare
        np.testing.assert_array_equal(t2n(dc.topk), idx)
        np.testing.assert_array_equal(t2n(ecnt), rcnt)
        np.testing.assert_array_equal(t2n(eidx)[rcnt == 1], ridx[rcnt == 1])
        np.testing.assert_array_equal(t2n(dc.n_valid), ref.n_valid)
        np.testing.assert_array_equal(t2n(d_birth), birth)
        np.testing.assert_array_equal(t2n(d_last), last)
        np.testing.assert_array_equal(t2n(d_freq), freq)
        evicted_any += int(rcnt.sum())
    assert evicted_any > 10
    for s in range(g.B * g.E):
        np.testing.assert_array_equal(dc.shard_host("K", s), ref.K_shards[s])


@pytest.mark.parametrize("S,cap", [(300, 200), (1000, 3), (64, 63), (700, 699)])
def test_policy_arrays_follow_a_compacting_eviction(S, cap):
    g = wl.Geometry(B=2, Hq=2, Hkv=2, D=16, E=3, S=S, k=2, dtype="bf16")
    case = wl.make_host_case(g, seed=81, n_valid="ragged", utility0="exp")
    case.n_valid[0, 0] = g.S
    case.n_valid[1, 2] = min(cap, g.S)                   # nothing to evict there
    rng = np.random.default_rng(15)
    birth, last, freq = random_state(rng, g.B, g.E, g.S, 900)
    dc = DeviceCase(case)
    d = [to_dev(a) for a in (birth, last, freq)]
    max_evict = g.S
    eidx = torch.full((g.B, g.E, max_evict), -1, device=DEV, dtype=torch.int32)
    ecnt = torch.zeros((g.B, g.E), device=DEV, dtype=torch.int32)
    pk.pikv_evict(dc.desc, dc.utility, dc.n_valid, cap, None, 0, eidx, ecnt, max_evict, True, dc.K_tab, dc.V_tab)
    pk.pikv_policy_compact(dc.desc, eidx, ecnt, max_evict, dc.n_valid, d[0], d[1], d[2])
    ref = case.clone()
    ridx, rcnt = orc.evict(ref.utility, ref.n_valid, cap, compact=True, K_shards=ref.K_shards, V_shards=ref.V_shards,
                           Hkv=g.Hkv, width=g.width, dtype=g.dtype, max_evict=max_evict)
    orc.policy_compact(ridx, rcnt, ref.n_valid, birth, last, freq)
    np.testing.assert_array_equal(t2n(ecnt), rcnt)
    n_after = t2n(dc.n_valid)
    np.testing.assert_array_equal(n_after, ref.n_valid)
    for got, want in zip(d, (birth, last, freq)):
        got = t2n(got)
        for b in range(g.B):
            for e in range(g.E):
                np.testing.assert_array_equal(got[b, e, :n_after[b, e]], want[b, e, :n_after[b, e]])
    assert rcnt.sum() > 0



@pytest.mark.parametrize("name", ["h2o_protect", "sl", "lru", "lru_plus"])
@pytest.mark.parametrize("spec", [
    dict(B=3, Hq=4, Hkv=2, D=64, E=8, S=48, k=2, dtype="bf16"),
    dict(B=2, Hq=8, Hkv=2, D=128, E=16, S=70, k=3, dtype="bf16"),          # matrix-core attention kernel
    dict(B=2, Hq=4, Hkv=4, D=128, E=8, S=40, k=2, dtype="bf16", rank=32),
    dict(B=33, Hq=2, Hkv=2, D=32, E=8, S=24, k=2, dtype="bf16"),           # many sequences
], ids=["d64", "gqa4_d128", "rank32", "b33_e8"])
def test_fused_step_with_a_policy_is_bit_identical_to_the_separate_calls(name, spec):
    """pikv_decode_step_policy against the sequence it is defined as: route, policy utility, evict,
    stamp, append, attend, tracked update - all state equal bit for bit over several steps."""
    g = wl.Geometry(**spec)
    case = wl.make_host_case(g, seed=91, utility0="exp", zipf_s=1.1)
    case.n_valid[:, 1] = g.S - 2
    policy = {"h2o_protect": pk.POLICY_H2O, "sl": pk.POLICY_SL, "lru": pk.POLICY_LRU, "lru_plus": pk.POLICY_LRU_PLUS}[name]
    protect = 6 if name == "h2o_protect" else 0
    lam, window, thr = 1.5, 12, 0.02
    rng = np.random.default_rng(16)
    birth, last, freq = random_state(rng, g.B, g.E, g.S, 20)
    dA, dB = DeviceCase(case), DeviceCase(case)
    sA = [to_dev(a) for a in (birth, last, freq)]
    sB = [to_dev(a) for a in (birth, last, freq)]
    u_pol = torch.zeros((g.B, g.E, g.S), device=DEV)
    eiA = torch.full((g.B, g.E, 1), -1, device=DEV, dtype=torch.int32)
    ecA = torch.full((g.B, g.E), -5, device=DEV, dtype=torch.int32)
    eiB, ecB = eiA.clone(), ecA.clone()
    evictions = 0
    for step in range(6):
        now = 21 + step
        qn = wl.draw_queries(g, 7000 + step)
        kn, vn = wl.draw_new_kv(g, 7100 + step)
        dkn, dvn = dev_storage(kn, g.dtype), dev_storage(vn, g.dtype)
        for d in (dA, dB):
            d.q.copy_(dev_storage(qn, g.dtype))
        args = pk.make_policy_args(policy, now, lam=lam, window=window, protect=protect, threshold=thr,
                                   birth=sA[0], last_access=sA[1], freq=sA[2])
        pk.pikv_decode_step_policy(dA.desc, dA.q, dA.W_r, dA.bias, dkn, dvn, dA.K_tab, dA.V_tab, dA.U_K, dA.U_V,
                                   dA.n_valid, dA.utility, g.k, pk.COMBINE_LSE, 0.0, 0.9, dA.topk, dA.gates,
                                   eiA, ecA, dA.y, dA.row_max, dA.row_norm, dA.scores, dA.slot_coef,
                                   dA.workspace, args)
        dB.route()
        pk.pikv_policy_utility(dB.desc, policy, dB.n_valid, now, lam, window, protect, sB[0], sB[1], sB[2],
                               dB.utility, u_pol)
        pk.pikv_evict(dB.desc, u_pol, dB.n_valid, g.S - 1, dB.topk, g.k, eiB, ecB, 1, False, None, None)
        pk.pikv_policy_stamp(dB.desc, dB.topk, g.k, eiB, ecB, 1, dB.n_valid, now, sB[0], sB[1], sB[2])
        pk.pikv_append(dB.desc, dkn, dvn, dB.topk, g.k, eiB, ecB, 1, dB.K_tab, dB.V_tab, dB.utility, dB.n_valid)
        dB.attend(combine=pk.COMBINE_LSE)
        pk.pikv_update_utility_tracked(dB.desc, dB.scores, dB.slot_coef, dB.n_valid, dB.topk, g.k, 0.9,
                                       dB.utility, thr, now, sB[1], sB[2])
        for nm in ("topk", "gates", "n_valid", "utility", "y", "K", "V"):
            a, b2 = getattr(dA, nm), getattr(dB, nm)
            if a.dtype == torch.bfloat16:
                a, b2 = a.view(torch.int16), b2.view(torch.int16)
            np.testing.assert_array_equal(t2n(a), t2n(b2), err_msg="%s differs at step %d" % (nm, step))
        for a, b2, nm in zip(sA, sB, ("birth", "last_access", "freq")):
            np.testing.assert_array_equal(t2n(a), t2n(b2), err_msg="%s differs at step %d" % (nm, step))
        np.testing.assert_array_equal(t2n(ecA), t2n(ecB))
        np.testing.assert_array_equal(t2n(eiA)[t2n(ecA) == 1], t2n(eiB)[t2n(ecB) == 1])
        evictions += int((t2n(ecA) == 1).sum())
    assert evictions > 0
    assert (t2n(sA[2]) != freq).any()            # accesses were counted
