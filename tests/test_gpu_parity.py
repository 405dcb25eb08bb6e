"""HIP path vs CPU oracle, element by element, on identical seeded inputs.

Bars: expert indices, evicted slots, appended rows: bit-exact.  Attention output:
|d| <= 2e-3 + 1e-2 |ref| (bf16 storage, fp32 accumulate) plus a relative-L2 bound of 1e-3;
utilities: rel 1e-4.  Sizes span several tiles, several splits and ragged tails.
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
from gpu_harness import (DEV, DeviceCase, assert_utility_close, ensure_route_margin, t2n,  # noqa: E402
                         y_tolerance_ok)


def oracle_step(case, idx, gates, combine, utility=None, decay=1.0, scale=0.0):
    g = case.geo
    return orc.attend(case.q, case.K_shards, case.V_shards, case.n_valid, idx, gates, Hkv=g.Hkv,
                      E=g.E, S=g.S, dtype=g.dtype, rank=g.rank, U_K=case.U_K, U_V=case.U_V,
                      combine=combine, scale=scale, utility=utility, decay=decay, want_prob=True)


# ---------------------------------------------------------------------- route
ROUTE_CASES = [
    # (rows-shape geometry, k)
    dict(B=1, Hq=4, Hkv=4, D=64, E=4, S=8, k=2, dtype="f32", per_head_routing=True),
    dict(B=8, Hq=32, Hkv=32, D=128, E=16, S=8, k=2, dtype="bf16"),
    dict(B=1, Hq=32, Hkv=8, D=128, E=16, S=8, k=4, dtype="bf16"),
    dict(B=32, Hq=32, Hkv=32, D=128, E=8, S=8, k=2, dtype="bf16"),
    dict(B=3, Hq=2, Hkv=1, D=16, E=5, S=8, k=3, dtype="f32"),
    dict(B=5, Hq=4, Hkv=4, D=32, E=64, S=8, k=7, dtype="bf16"),
    dict(B=2, Hq=8, Hkv=8, D=64, E=1, S=8, k=1, dtype="bf16"),
    dict(B=4, Hq=8, Hkv=8, D=64, E=33, S=8, k=33, dtype="f32"),
]


@pytest.mark.parametrize("spec", ROUTE_CASES, ids=lambda s: "E%d_k%d_%s_B%d" % (s["E"], s["k"], s["dtype"], s["B"]))
@pytest.mark.parametrize("with_bias", [False, True])
def test_route_matches_oracle(spec, with_bias):
    g = wl.Geometry(**spec)
    case = wl.make_host_case(g, seed=3, w_sigma=1.0 if g.dtype == "f32" else 0.02,
                             zipf_s=1.1 if with_bias else 0.0)
    ensure_route_margin(case, g.k)
    dc = DeviceCase(case)
    dc.route()
    x = np.ascontiguousarray(case.q.reshape(g.route_rows, g.d_r))
    idx, gates, probs = orc.route(x, case.W_r, g.k, bias=case.bias, dtype=g.dtype)
    np.testing.assert_array_equal(t2n(dc.topk), idx)
    np.testing.assert_allclose(t2n(dc.gates), gates, rtol=2e-5, atol=1e-7)
    np.testing.assert_allclose(t2n(dc.probs), probs, rtol=2e-5, atol=1e-7)


def test_route_exact_ties_lower_index_first():
    rng = np.random.default_rng(6)
    rows, d_r = 64, 32
    x = rng.integers(-3, 4, size=(rows, d_r)).astype(np.float32)
    Wb = rng.integers(-2, 3, size=(d_r, 4)).astype(np.float32)
    W = np.ascontiguousarray(np.concatenate([Wb, Wb[:, [1, 3]], Wb[:, [0]], Wb], axis=1))   # E = 11
    x[0] = 0
    for dtype in ("f32", "bf16"):
        xs, Ws = wl.encode(x, dtype), wl.encode(W, dtype)
        for k in (1, 3, 6, 11):
            idx, gates, _ = orc.route(xs, Ws, k, dtype=dtype)
            from gpu_harness import dev_storage
            tk = torch.zeros((rows, k), device=DEV, dtype=torch.int32)
            tg = torch.zeros((rows, k), device=DEV)
            pk.pikv_route(dev_storage(xs, dtype), dev_storage(Ws, dtype), None, rows, d_r, 11, k, tk, tg)
            np.testing.assert_array_equal(t2n(tk), idx)
            np.testing.assert_allclose(t2n(tg), gates, rtol=2e-5)


def test_round_robin_router_matches_oracle_and_feeds_attention():
    g = wl.Geometry(B=5, Hq=4, Hkv=2, D=64, E=7, S=90, k=3, dtype="bf16")
    case = wl.make_host_case(g, seed=17, n_valid="ragged")
    dc = DeviceCase(case)
    for step in (0, 4, 123456789):
        pk.pikv_route_round_robin(g.B, g.E, g.k, step, dc.topk, dc.gates)
        idx, gates = orc.route_round_robin(g.B, g.E, g.k, step)
        np.testing.assert_array_equal(t2n(dc.topk), idx)
        np.testing.assert_array_equal(t2n(dc.gates), gates)
    ref = oracle_step(case, idx, gates, orc.COMBINE_LOCAL)
    dc.attend(combine=pk.COMBINE_LOCAL)
    ok, emax, l2 = y_tolerance_ok(t2n(dc.y), ref["y"], g.dtype)
    assert ok, (emax, l2)
    with pytest.raises(pk.PikvError):
        pk.pikv_route_round_robin(g.B, g.E, g.E + 1, 0, dc.topk, dc.gates)


# ------------------------------------------------------------------ attention
ATTN_CASES = {
    # config 1 itself: per-head routing, fp32
    "c1_tiny_f32": (dict(B=1, Hq=4, Hkv=4, D=64, E=4, S=256, k=2, dtype="f32", per_head_routing=True), "full"),
    # scaled config 2: G=1, bf16, several splits and a ragged tail
    "c2_scaled": (dict(B=2, Hq=4, Hkv=4, D=128, E=6, S=700, k=2, dtype="bf16"), "ragged"),
    # scaled config 3: GQA group of 4, k=4
    "c3_scaled": (dict(B=1, Hq=8, Hkv=2, D=128, E=8, S=1100, k=4, dtype="bf16"), "ragged"),
    "gqa2": (dict(B=2, Hq=4, Hkv=2, D=64, E=4, S=300, k=2, dtype="bf16"), "ragged"),
    "gqa8": (dict(B=1, Hq=8, Hkv=1, D=128, E=4, S=260, k=2, dtype="bf16"), "full"),
    "gqa3_generic": (dict(B=1, Hq=6, Hkv=2, D=64, E=4, S=150, k=3, dtype="bf16"), "ragged"),
    # matrix-core grouped-query kernel (bf16, D=128): odd group sizes, the 16-head limit, short tails
    "gqa3_d128": (dict(B=2, Hq=6, Hkv=2, D=128, E=4, S=333, k=2, dtype="bf16"), "ragged"),
    "gqa16_d128": (dict(B=1, Hq=16, Hkv=1, D=128, E=3, S=1500, k=2, dtype="bf16"), "ragged"),
    "gqa5_d128_tiny": (dict(B=1, Hq=5, Hkv=1, D=128, E=2, S=7, k=2, dtype="bf16"), "full"),
    # more than 16 rows per kv head: two and four 16-row tiles sharing every K/V load
    "gqa32_two_row_tiles": (dict(B=1, Hq=32, Hkv=1, D=128, E=2, S=70, k=1, dtype="bf16"), "full"),
    "gqa17_d128": (dict(B=2, Hq=34, Hkv=2, D=128, E=3, S=400, k=2, dtype="bf16"), "ragged"),
    "gqa48_d128": (dict(B=1, Hq=96, Hkv=2, D=128, E=3, S=700, k=2, dtype="bf16"), "ragged"),
    "gqa64_d128": (dict(B=1, Hq=128, Hkv=2, D=128, E=4, S=1300, k=3, dtype="bf16"), "ragged"),
    # scaled config 5: rank-32 codes
    "c5_scaled": (dict(B=2, Hq=4, Hkv=4, D=128, E=6, S=900, k=2, dtype="bf16", rank=32), "ragged"),
    "rank16_gqa4": (dict(B=1, Hq=8, Hkv=2, D=64, E=4, S=520, k=2, dtype="bf16", rank=16), "ragged"),
    "rank64_f32": (dict(B=1, Hq=2, Hkv=2, D=128, E=3, S=130, k=2, dtype="f32", rank=64), "full"),
    "f32_d128": (dict(B=1, Hq=2, Hkv=1, D=128, E=3, S=100, k=3, dtype="f32"), "ragged"),
    "d32_bf16": (dict(B=2, Hq=2, Hkv=2, D=32, E=4, S=515, k=2, dtype="bf16"), "ragged"),
    "d16_bf16_perhead": (dict(B=2, Hq=4, Hkv=2, D=16, E=4, S=1030, k=2, dtype="bf16", per_head_routing=True), "ragged"),
    "k_equals_E": (dict(B=1, Hq=4, Hkv=4, D=64, E=4, S=129, k=4, dtype="bf16"), "ragged"),
    "one_slot": (dict(B=1, Hq=2, Hkv=2, D=64, E=2, S=1, k=2, dtype="bf16"), "full"),
    # the limits: longest shards, most query heads, most experts
    "long_shard_70k": (dict(B=1, Hq=4, Hkv=2, D=128, E=2, S=70000, k=2, dtype="bf16"), "ragged"),
    "long_shard_g1_40k": (dict(B=1, Hq=2, Hkv=2, D=64, E=2, S=40000, k=1, dtype="bf16"), "full"),
    "hq256": (dict(B=1, Hq=256, Hkv=32, D=64, E=2, S=64, k=2, dtype="bf16"), "ragged"),
    "e64_k64": (dict(B=1, Hq=2, Hkv=2, D=32, E=64, S=40, k=64, dtype="bf16"), "ragged"),
    # the utility kernel's shape for hundreds of query rows: heads chosen per head (an expert's
    # active heads differ in number, down to none), slot tiles with a ragged end
    "hq160_perhead": (dict(B=2, Hq=160, Hkv=4, D=32, E=3, S=150, k=2, dtype="bf16", per_head_routing=True), "ragged"),
    "hq128_k1": (dict(B=1, Hq=128, Hkv=2, D=128, E=5, S=333, k=1, dtype="bf16"), "ragged"),
}


def random_selection(g, seed):
    rng = np.random.default_rng(seed)
    idx = np.stack([rng.permutation(g.E)[:g.k] for _ in range(g.route_rows)]).astype(np.int32)
    gates = rng.random((g.route_rows, g.k)).astype(np.float32) + 0.05
    gates /= gates.sum(-1, keepdims=True)
    return idx, gates.astype(np.float32)


@pytest.mark.parametrize("name", sorted(ATTN_CASES))
@pytest.mark.parametrize("combine", [orc.COMBINE_LSE, orc.COMBINE_LOCAL], ids=["lse", "local"])
@pytest.mark.parametrize("use_gates", [True, False], ids=["gates", "mask"])
def test_attention_and_utility_match_oracle(name, combine, use_gates):
    spec, nv = ATTN_CASES[name]
    g = wl.Geometry(**spec)
    case = wl.make_host_case(g, seed=11, kv="lognormal_token", n_valid=nv, utility0="exp")
    idx, gates = random_selection(g, 5)
    if not use_gates:
        gates = None
    u_ref = case.utility.copy()
    ref = oracle_step(case, idx, gates, combine, utility=u_ref, decay=0.9)

    dc = DeviceCase(case)
    d_idx = torch.from_numpy(idx).to(DEV)
    d_gates = None if gates is None else torch.from_numpy(gates).to(DEV)
    dc.attend(topk=d_idx, gates=d_gates, combine=combine)
    dc.update_utility(0.9, topk=d_idx)

    y = t2n(dc.y)
    ok, emax, l2 = y_tolerance_ok(y, ref["y"], g.dtype)
    assert ok, "y mismatch: max abs %.3e, rel L2 %.3e" % (emax, l2)
    np.testing.assert_allclose(t2n(dc.row_max), ref["row_max"], rtol=1e-4, atol=1e-5)
    np.testing.assert_allclose(t2n(dc.row_norm), ref["row_norm"], rtol=1e-4, atol=1e-9)
    assert_utility_close(t2n(dc.utility), u_ref)
    # per-entry probabilities rebuilt from the emitted scores and (shift, coef)
    sc, co = t2n(dc.scores).astype(np.float64), t2n(dc.slot_coef).astype(np.float64)
    for b in range(g.B):
        for h in range(g.Hq):
            row = b * g.Hq + h if g.per_head_routing else b
            for j in range(g.k):
                n = case.n_valid[b, idx[row, j]]
                p = co[b, h, j, 1] * np.exp(sc[b, h, j, :n] - co[b, h, j, 0])
                np.testing.assert_allclose(p, ref["prob"][b, h, j, :n], rtol=1e-4, atol=1e-10)


@pytest.mark.parametrize("spec", [
    dict(B=2, Hq=16, Hkv=2, D=128, E=4, S=300, k=2, dtype="bf16", tq=4),      # 8 rows per kv head
    dict(B=1, Hq=64, Hkv=2, D=128, E=4, S=500, k=2, dtype="bf16", tq=8),      # 32 rows: two row tiles
    dict(B=2, Hq=128, Hkv=2, D=128, E=3, S=200, k=2, dtype="bf16", tq=16),    # 64 rows: four row tiles
    dict(B=1, Hq=72, Hkv=3, D=128, E=3, S=150, k=3, dtype="bf16", tq=6),      # 24 rows, three kv heads
], ids=["tq4", "tq8", "tq16", "tq6_kv3"])
@pytest.mark.parametrize("combine", [orc.COMBINE_LSE, orc.COMBINE_LOCAL], ids=["lse", "local"])
def test_multi_query_step_in_token_major_layout(spec, combine):
    """Draft queries of a multi-query step in their natural layout, q [B, tq, heads, D] with
    desc.tq = tq: routing by the tile's first query, attention of every (draft, head) row over the
    selected shards, outputs back in [B, tq, heads] order, utilities summed over all rows.  The
    oracle sees the same rows as Hq = tq * heads plain query heads in kv-head-first order."""
    from gpu_harness import dev_storage
    g = wl.Geometry(token_major=True, **spec)
    case = wl.make_host_case(g, seed=71, n_valid="ragged", utility0="exp", w_sigma=0.02)
    perm = wl.token_major_rows(g.Hq, g.Hkv, g.tq)           # internal row -> caller row
    q_caller = np.empty_like(case.q)
    q_caller[:, perm] = case.q                               # the caller's [B, tq*heads, D]
    # the router sees the caller's flat vector
    probe = case.clone()
    probe.q = q_caller
    ensure_route_margin(probe, g.k)
    q_caller = probe.q
    case.q = np.ascontiguousarray(q_caller[:, perm])        # oracle order of the same rows
    dc = DeviceCase(case)
    dc.q = dev_storage(q_caller, g.dtype)
    dc.desc = pk.make_desc(g.B, g.Hq, g.Hkv, g.D, g.E, g.S, dtype=pk.binding.BF16, stride_h=dc.stride_h,
                           stride_s=dc.stride_s, tq=g.tq)
    dc.route()
    x = np.ascontiguousarray(wl.routing_rows(g, q_caller))   # the tile's first query routes the step
    assert x.shape == (g.B, g.Hq // g.tq * g.D)
    np.testing.assert_array_equal(x, q_caller[:, :g.Hq // g.tq].reshape(g.B, -1))
    idx, gates, _ = orc.route(x, case.W_r, g.k, dtype=g.dtype)
    np.testing.assert_array_equal(t2n(dc.topk), idx)
    dc.attend(combine=combine)
    dc.update_utility(0.9)
    u_ref = case.utility.copy()
    ref = oracle_step(case, idx, t2n(dc.gates), combine, utility=u_ref, decay=0.9)
    y = t2n(dc.y)[:, perm]                                   # back to the oracle's row order
    ok, emax, l2 = y_tolerance_ok(y, ref["y"], g.dtype)
    assert ok, (emax, l2)
    np.testing.assert_allclose(t2n(dc.row_max)[:, perm], ref["row_max"], rtol=1e-4, atol=1e-5)
    np.testing.assert_allclose(t2n(dc.row_norm)[:, perm], ref["row_norm"], rtol=1e-4, atol=1e-9)
    assert_utility_close(t2n(dc.utility), u_ref)


def test_library_opened_before_torch_still_launches():
    """A caller may load the binding's library before it ever imports torch; both must end up on
    one HIP runtime (a kernel launched through a second copy fails on torch's streams).  Runs in
    a fresh interpreter, because this process has imported torch long ago."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = (
        "import sys; sys.path.insert(0, %r)\n"
        "import paper_2508_06526_amd as pk\n"
        "assert pk.load_library().pikv_version() >= 300\n"
        "import torch\n"
        "x = torch.eye(8, device='cuda:0'); W = torch.eye(8, device='cuda:0')\n"
        "idx = torch.zeros((8, 1), device='cuda:0', dtype=torch.int32); g = torch.zeros((8, 1), device='cuda:0')\n"
        "pk.pikv_route(x, W, None, 8, 8, 8, 1, idx, g)\n"
        "torch.cuda.synchronize()\n"
        "assert idx.flatten().tolist() == list(range(8)), idx\n"
        "print('ok')\n" % root)
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=110)
    assert r.returncode == 0 and "ok" in r.stdout, (r.stdout[-500:], r.stderr[-1500:])


def test_multi_query_layout_is_refused_where_no_kernel_takes_it():
    fake = torch.zeros(64, device=DEV)
    for kw in (dict(D=64), dict(rank=32), dict(dtype=pk.binding.F32)):     # only bf16 rows of 128 values
        args = dict(D=128, rank=0, dtype=pk.binding.BF16)
        args.update(kw)
        desc = pk.make_desc(1, 16, 2, args["D"], 4, 64, rank=args["rank"], dtype=args["dtype"], tq=4)
        ws = torch.empty(1 << 20, device=DEV, dtype=torch.uint8)
        with pytest.raises(pk.PikvError) as err:
            pk.pikv_sharded_attn(desc, fake, fake, fake, fake, fake, fake, fake, None, 2, pk.COMBINE_LSE, 0.0,
                                 fake, None, None, None, None, ws)
        assert err.value.status == -2


def random_geometry(rng):
    D = int(rng.choice([16, 32, 64, 128]))
    dtype = str(rng.choice(["bf16", "bf16", "f32"]))
    rank = int(rng.choice([0, 0, 16, 32, 64]))
    if rank >= D:
        rank = 0
    Hkv = int(rng.choice([1, 2, 3, 4]))
    G = int(rng.choice([1, 1, 2, 3, 4, 5, 8, 16, 24, 40]))
    E = int(rng.integers(1, 10))
    k = int(rng.integers(1, E + 1))
    per_head = bool(rng.random() < 0.25)
    return dict(B=int(rng.integers(1, 4)), Hq=Hkv * G, Hkv=Hkv, D=D, E=E, S=int(rng.integers(1, 700)), k=k,
                dtype=dtype, rank=rank, per_head_routing=per_head)


@pytest.mark.parametrize("seed", range(24))
def test_attention_on_random_geometries(seed):
    """Seeded sweep over shapes nobody hand-picked: head grouping, widths, code ranks, shard counts,
    ragged fills, both combine modes, gates or mask, split counts forced or chosen."""
    rng = np.random.default_rng(1000 + seed)
    g = wl.Geometry(**random_geometry(rng))
    case = wl.make_host_case(g, seed=seed, kv="lognormal_token", n_valid=str(rng.choice(["ragged", "full"])),
                             utility0="exp")
    idx, gates = random_selection(g, 50 + seed)
    if rng.random() < 0.3:
        gates = None
    combine = int(rng.choice([orc.COMBINE_LSE, orc.COMBINE_LOCAL]))
    u_ref = case.utility.copy()
    ref = oracle_step(case, idx, gates, combine, utility=u_ref, decay=0.7)
    forced = int(rng.choice([0, 0, 1, 3, 7]))
    pk.pikv_set_attn_split(forced)
    try:
        dc = DeviceCase(case)
        d_idx = torch.from_numpy(idx).to(DEV)
        d_gates = None if gates is None else torch.from_numpy(gates).to(DEV)
        dc.attend(topk=d_idx, gates=d_gates, combine=combine)
        dc.update_utility(0.7, topk=d_idx)
        y, u = t2n(dc.y), t2n(dc.utility)
    finally:
        pk.pikv_set_attn_split(0)
    ok, emax, l2 = y_tolerance_ok(y, ref["y"], g.dtype)
    assert ok, "geometry %s: max abs %.3e, rel L2 %.3e" % (g, emax, l2)
    np.testing.assert_allclose(t2n(dc.row_max), ref["row_max"], rtol=1e-4, atol=1e-5)
    assert_utility_close(u, u_ref)


def test_attention_is_bitwise_repeatable():
    spec, nv = ATTN_CASES["c3_scaled"]
    g = wl.Geometry(**spec)
    case = wl.make_host_case(g, seed=12, n_valid=nv)
    idx, gates = random_selection(g, 6)
    dc = DeviceCase(case)
    d_idx, d_gates = torch.from_numpy(idx).to(DEV), torch.from_numpy(gates).to(DEV)
    outs = []
    for _ in range(2):
        dc.utility.zero_()
        dc.attend(topk=d_idx, gates=d_gates)
        dc.update_utility(1.0, topk=d_idx)
        outs.append((t2n(dc.y), t2n(dc.utility)))
    np.testing.assert_array_equal(outs[0][0], outs[1][0])
    np.testing.assert_array_equal(outs[0][1], outs[1][1])


def test_strided_shards_and_explicit_scale():
    g = wl.Geometry(B=1, Hq=4, Hkv=2, D=64, E=3, S=200, k=2, dtype="bf16")
    case = wl.make_host_case(g, seed=13, n_valid="ragged")
    idx, gates = random_selection(g, 7)
    ref = oracle_step(case, idx, gates, orc.COMBINE_LSE, scale=0.2)
    dc = DeviceCase(case, stride_pad=(8, 5))
    dc.attend(topk=torch.from_numpy(idx).to(DEV), gates=torch.from_numpy(gates).to(DEV), scale=0.2,
              want_scores=False)
    ok, emax, l2 = y_tolerance_ok(t2n(dc.y), ref["y"], g.dtype)
    assert ok, (emax, l2)


def test_all_selected_shards_empty_gives_zero_and_leaves_utility():
    g = wl.Geometry(B=2, Hq=4, Hkv=4, D=64, E=4, S=64, k=2, dtype="bf16")
    case = wl.make_host_case(g, seed=14, utility0="exp")
    case.n_valid[0, :] = 0
    case.n_valid[1, 2] = 0
    idx = np.array([[0, 1], [2, 3]], np.int32)
    u_ref = case.utility.copy()
    ref = oracle_step(case, idx, None, orc.COMBINE_LSE, utility=u_ref, decay=0.5)
    dc = DeviceCase(case)
    d_idx = torch.from_numpy(idx).to(DEV)
    dc.attend(topk=d_idx, gates=None)
    dc.update_utility(0.5, topk=d_idx)
    y = t2n(dc.y)
    assert (y[0] == 0).all()
    ok, emax, l2 = y_tolerance_ok(y, ref["y"], g.dtype)
    assert ok, (emax, l2)
    assert_utility_close(t2n(dc.utility), u_ref)
    np.testing.assert_array_equal(t2n(dc.utility)[0], case.utility[0])


# ---------------------------------------------------------------- evict / append
def run_gpu_evict(g, u, n, capacity, sel=None, max_evict=None, compact=False, case=None):
    dt = g.dtype
    if case is None:
        case = wl.make_host_case(g, seed=1)
    case = case.clone()
    case.utility, case.n_valid = u.copy(), n.copy()
    dc = DeviceCase(case)
    if max_evict is None:
        max_evict = max(1, g.S - capacity)
    eidx = torch.full((g.B, g.E, max_evict), -1, device=DEV, dtype=torch.int32)
    ecnt = torch.full((g.B, g.E), -7, device=DEV, dtype=torch.int32)
    d_sel = None if sel is None else torch.from_numpy(sel).to(DEV)
    pk.pikv_evict(dc.desc, dc.utility, dc.n_valid, capacity, d_sel, 0 if sel is None else sel.shape[1],
                  eidx, ecnt, max_evict, compact, dc.K_tab if compact else None,
                  dc.V_tab if compact else None)
    return dc, t2n(eidx), t2n(ecnt)


@pytest.mark.parametrize("S,capacity", [(256, 192), (1000, 1), (16, 6), (2048, 2047), (5000, 4096), (300, 0),
                                        (3000, 2000), (12000, 9000), (20000, 100), (40000, 30000), (1001, 700), (255, 100)])
@pytest.mark.parametrize("ties", [False, True], ids=["distinct", "ties"])
def test_evict_matches_oracle_bit_exact(S, capacity, ties):
    g = wl.Geometry(B=2, Hq=2, Hkv=2, D=16, E=3, S=S, k=2, dtype="bf16")
    rng = np.random.default_rng(S + capacity)
    if ties:
        u = (rng.integers(0, 6, size=(g.B, g.E, S)) / 8).astype(np.float32)
    else:
        u = (rng.exponential(1.0, size=(g.B, g.E, S)) / S).astype(np.float32)
    n = rng.integers(max(0, capacity - 3), S + 1, size=(g.B, g.E)).astype(np.int32)
    n[0, 0] = S
    u_ref, n_ref = u.copy(), n.copy()
    ridx, rcnt = orc.evict(u_ref, n_ref, capacity, max_evict=max(1, S - capacity))
    dc, eidx, ecnt = run_gpu_evict(g, u, n, capacity)
    np.testing.assert_array_equal(ecnt, rcnt)
    for b in range(g.B):
        for e in range(g.E):
            np.testing.assert_array_equal(eidx[b, e, :rcnt[b, e]], ridx[b, e, :rcnt[b, e]])
    np.testing.assert_array_equal(t2n(dc.n_valid), n_ref)
    np.testing.assert_array_equal(t2n(dc.utility), u_ref)


def test_evict_special_values_and_selection_list():
    g = wl.Geometry(B=2, Hq=2, Hkv=2, D=16, E=4, S=64, k=2, dtype="bf16")
    rng = np.random.default_rng(3)
    u = rng.standard_normal((g.B, g.E, g.S)).astype(np.float32)       # negative utilities too
    u[0, 1, ::3] = 0.0
    u[0, 1, 1::6] = -0.0
    u[1, 2, :] = 0.25                                                  # all equal
    n = np.full((g.B, g.E), g.S, np.int32)
    sel = np.array([[1, 3], [2, 0]], np.int32)
    mask = np.zeros((g.B, g.E), np.int32)
    for b in range(g.B):
        mask[b, sel[b]] = 1
    u_ref, n_ref = u.copy(), n.copy()
    ridx, rcnt = orc.evict(u_ref, n_ref, 40, shard_mask=mask, max_evict=24)
    dc, eidx, ecnt = run_gpu_evict(g, u, n, 40, sel=sel, max_evict=24)
    np.testing.assert_array_equal(ecnt, rcnt)
    np.testing.assert_array_equal(eidx[mask == 1], ridx[mask == 1])
    np.testing.assert_array_equal(t2n(dc.n_valid), n_ref)
    # more to evict than max_evict: shard untouched, count -1
    dc, eidx, ecnt = run_gpu_evict(g, u, n, 10, max_evict=5)
    assert (ecnt == -1).all() and (t2n(dc.n_valid) == g.S).all()


@pytest.mark.parametrize("spec", [
    dict(B=1, Hq=4, Hkv=4, D=64, E=4, S=256, k=2, dtype="f32", per_head_routing=True),   # config 1: 256 -> 192
    dict(B=2, Hq=4, Hkv=2, D=128, E=3, S=700, k=2, dtype="bf16"),
    dict(B=1, Hq=2, Hkv=2, D=128, E=2, S=300, k=2, dtype="bf16", rank=32),
    dict(B=1, Hq=2, Hkv=2, D=128, E=2, S=3000, k=2, dtype="bf16"),       # many passes of the row mover
    dict(B=1, Hq=2, Hkv=1, D=128, E=2, S=600, k=1, dtype="f32"),         # 512-byte rows
    dict(B=1, Hq=2, Hkv=2, D=16, E=2, S=2500, k=1, dtype="bf16"),        # 32-byte rows
], ids=["c1", "bf16_d128", "rank32", "bf16_s3000", "f32_d128", "bf16_d16"])
def test_evict_with_compaction_moves_rows_like_oracle(spec):
    g = wl.Geometry(**spec)
    case = wl.make_host_case(g, seed=21, n_valid="ragged", utility0="exp")
    case.n_valid[0, 0] = g.S
    capacity = (g.S * 3) // 4
    ref = case.clone()
    ridx, rcnt = orc.evict(ref.utility, ref.n_valid, capacity, compact=True, K_shards=ref.K_shards,
                           V_shards=ref.V_shards, Hkv=g.Hkv, width=g.width, dtype=g.dtype)
    dc, eidx, ecnt = run_gpu_evict(g, case.utility, case.n_valid, capacity, compact=True, case=case)
    np.testing.assert_array_equal(ecnt, rcnt)
    n_new = t2n(dc.n_valid)
    np.testing.assert_array_equal(n_new, ref.n_valid)
    u = t2n(dc.utility)
    for b in range(g.B):
        for e in range(g.E):
            s, nn = b * g.E + e, n_new[b, e]
            np.testing.assert_array_equal(eidx[b, e, :rcnt[b, e]], ridx[b, e, :rcnt[b, e]])
            np.testing.assert_array_equal(u[b, e, :nn], ref.utility[b, e, :nn])
            np.testing.assert_array_equal(dc.shard_host("K", s)[:, :nn], ref.K_shards[s][:, :nn])
            np.testing.assert_array_equal(dc.shard_host("V", s)[:, :nn], ref.V_shards[s][:, :nn])


def test_append_matches_oracle_bit_exact():
    g = wl.Geometry(B=3, Hq=4, Hkv=2, D=128, E=4, S=50, k=2, dtype="bf16")
    case = wl.make_host_case(g, seed=22, n_valid="ragged", utility0="exp")
    case.n_valid[1, 1] = g.S                                # a full shard: entry dropped
    idx = np.array([[0, 2], [1, 3], [3, 0]], np.int32)
    kn, vn = wl.draw_new_kv(g, 5)
    from gpu_harness import dev_storage
    dc = DeviceCase(case)
    pk.pikv_append(dc.desc, dev_storage(kn, g.dtype), dev_storage(vn, g.dtype),
                   torch.from_numpy(idx).to(DEV), g.k, None, None, 0, dc.K_tab, dc.V_tab,
                   dc.utility, dc.n_valid)
    ref = case.clone()
    # the oracle reports a full shard as an error; the library drops the entry for that shard
    idx_ok = idx.copy()
    ref_n_full = ref.n_valid.copy()
    for b in range(g.B):
        sel = [e for e in idx[b] if ref.n_valid[b, e] < g.S]
        for e in sel:
            one = np.array([[e]], np.int32)
            orc.append(np.ascontiguousarray(kn[b:b + 1]), np.ascontiguousarray(vn[b:b + 1]), one,
                       ref.K_shards[b * g.E:(b + 1) * g.E], ref.V_shards[b * g.E:(b + 1) * g.E],
                       ref.utility[b:b + 1], ref.n_valid[b:b + 1], dtype=g.dtype)
    np.testing.assert_array_equal(t2n(dc.n_valid), ref.n_valid)
    np.testing.assert_array_equal(t2n(dc.utility), ref.utility)
    for s in range(g.B * g.E):
        np.testing.assert_array_equal(dc.shard_host("K", s), ref.K_shards[s])
        np.testing.assert_array_equal(dc.shard_host("V", s), ref.V_shards[s])
    assert ref.n_valid[1, 1] == g.S and idx_ok is not None and ref_n_full is not None


# --------------------------------------------------------- streaming (config 4, scaled)
def test_streaming_steps_route_evict_append_attend_update():
    """Each step: route -> evict the min-utility entry of every selected full shard ->
    append the new token there -> attend -> utility with decay 0.9.  The GPU carries its own
    state; at every step its selections and evicted slots must equal the oracle's applied
    to the GPU's own pre-step bits, and the free-running oracle state must stay within
    tolerance."""
    g = wl.Geometry(B=4, Hq=4, Hkv=4, D=64, E=4, S=96, k=2, dtype="bf16")
    case = wl.make_host_case(g, seed=31, utility0="exp")
    case.n_valid[:, 0] = g.S - 2                      # some shards still have room
    from gpu_harness import dev_storage
    dc = DeviceCase(case)
    eidx = torch.full((g.B, g.E, 1), -1, device=DEV, dtype=torch.int32)
    ecnt = torch.zeros((g.B, g.E), device=DEV, dtype=torch.int32)
    ref = case.clone()
    for step in range(12):
        qn = wl.draw_queries(g, 500 + step)
        probe = case.clone()
        probe.q = qn
        ensure_route_margin(probe, g.k)
        qn = probe.q
        kn, vn = wl.draw_new_kv(g, 900 + step)
        # --- GPU
        dc.q.copy_(dev_storage(qn, g.dtype))
        u_before, n_before = t2n(dc.utility), t2n(dc.n_valid)
        dc.route()
        pk.pikv_evict(dc.desc, dc.utility, dc.n_valid, g.S - 1, dc.topk, g.k, eidx, ecnt, 1, False,
                      None, None)
        pk.pikv_append(dc.desc, dev_storage(kn, g.dtype), dev_storage(vn, g.dtype), dc.topk, g.k,
                       eidx, ecnt, 1, dc.K_tab, dc.V_tab, dc.utility, dc.n_valid)
        dc.attend(combine=pk.COMBINE_LSE)
        dc.update_utility(0.9)
        # --- oracle, free running
        x = np.ascontiguousarray(qn.reshape(g.route_rows, g.d_r))
        idx, gates, _ = orc.route(x, ref.W_r, g.k, dtype=g.dtype)
        np.testing.assert_array_equal(t2n(dc.topk), idx)
        mask = np.zeros((g.B, g.E), np.int32)
        for b in range(g.B):
            mask[b, idx[b]] = 1
        # evict parity on identical bits: the oracle applied to the GPU's own pre-step state
        ub, nb = u_before.copy(), n_before.copy()
        pidx, pcnt = orc.evict(ub, nb, g.S - 1, shard_mask=mask, max_evict=1)
        np.testing.assert_array_equal(t2n(ecnt), pcnt)
        np.testing.assert_array_equal(t2n(eidx)[pcnt == 1], pidx[pcnt == 1])
        ridx, rcnt = orc.evict(ref.utility, ref.n_valid, g.S - 1, shard_mask=mask, max_evict=1)
        np.testing.assert_array_equal(rcnt, pcnt)
        assert (ridx[rcnt == 1] == pidx[pcnt == 1]).all(), "free-running oracle diverged at step %d" % step
        orc.append(kn, vn, idx, ref.K_shards, ref.V_shards, ref.utility, ref.n_valid, dtype=g.dtype,
                   reuse_idx=ridx, reuse_cnt=rcnt)
        ref.q = qn
        out = oracle_step(ref, idx, gates, orc.COMBINE_LSE, utility=ref.utility, decay=0.9)
        ok, emax, l2 = y_tolerance_ok(t2n(dc.y), out["y"], g.dtype)
        assert ok, (step, emax, l2)
        assert_utility_close(t2n(dc.utility), ref.utility)
        np.testing.assert_array_equal(t2n(dc.n_valid), ref.n_valid)
        assert (ref.n_valid <= g.S).all()
    for s in range(g.B * g.E):
        np.testing.assert_array_equal(dc.shard_host("K", s), ref.K_shards[s])


# ------------------------------------------------------------------- fused decode step
@pytest.mark.parametrize("spec", [
    dict(B=4, Hq=4, Hkv=4, D=64, E=8, S=96, k=2, dtype="bf16"),
    dict(B=2, Hq=8, Hkv=2, D=128, E=16, S=200, k=4, dtype="bf16"),
    dict(B=3, Hq=4, Hkv=4, D=128, E=8, S=64, k=5, dtype="bf16", rank=32),
    dict(B=2, Hq=4, Hkv=2, D=64, E=4, S=50, k=2, dtype="f32"),
    dict(B=2, Hq=8, Hkv=2, D=128, E=12, S=120, k=3, dtype="bf16"),       # W_r rows of 24 bytes: generic router
    dict(B=1, Hq=4, Hkv=4, D=64, E=2, S=70, k=2, dtype="bf16"),          # ... of 4 bytes
    # many sequences: more blocks in the step's first kernel than the GPU has compute units
    dict(B=36, Hq=4, Hkv=4, D=64, E=8, S=40, k=2, dtype="bf16"),
    dict(B=90, Hq=2, Hkv=2, D=32, E=3, S=24, k=2, dtype="f32"),
], ids=["g1", "gqa4", "rank32_k5", "f32", "e12", "e2", "b36_e8", "b90_e3_f32"])
def test_fused_decode_step_equals_separate_calls_and_oracle(spec):
    """pikv_decode_step (3 launches) vs the five separate calls (bit-identical state) vs oracle."""
    from gpu_harness import dev_storage
    g = wl.Geometry(**spec)
    case = wl.make_host_case(g, seed=41, utility0="exp", zipf_s=1.1)
    case.n_valid[:, 0] = g.S - 3                       # a shard with room
    dA, dB = DeviceCase(case), DeviceCase(case)
    eiA = torch.full((g.B, g.E, 1), -1, device=DEV, dtype=torch.int32)
    ecA = torch.full((g.B, g.E), -5, device=DEV, dtype=torch.int32)
    eiB, ecB = eiA.clone(), ecA.clone()
    ref = case.clone()
    for step in range(6):
        probe = case.clone()
        probe.q = wl.draw_queries(g, 700 + step)
        ensure_route_margin(probe, g.k)
        qn = probe.q
        kn, vn = wl.draw_new_kv(g, 800 + step)
        dkn, dvn = dev_storage(kn, g.dtype), dev_storage(vn, g.dtype)
        for d in (dA, dB):
            d.q.copy_(dev_storage(qn, g.dtype))
        # A: fused
        pk.pikv_decode_step(dA.desc, dA.q, dA.W_r, dA.bias, dkn, dvn, dA.K_tab, dA.V_tab, dA.U_K, dA.U_V,
                            dA.n_valid, dA.utility, g.k, pk.COMBINE_LSE, 0.0, 0.9, dA.topk, dA.gates,
                            eiA, ecA, dA.y, dA.row_max, dA.row_norm, dA.scores, dA.slot_coef, dA.workspace)
        # B: separate calls
        dB.route()
        pk.pikv_evict(dB.desc, dB.utility, dB.n_valid, g.S - 1, dB.topk, g.k, eiB, ecB, 1, False, None, None)
        pk.pikv_append(dB.desc, dkn, dvn, dB.topk, g.k, eiB, ecB, 1, dB.K_tab, dB.V_tab, dB.utility, dB.n_valid)
        dB.attend(combine=pk.COMBINE_LSE)
        dB.update_utility(0.9)
        for name in ("topk", "gates", "n_valid", "utility", "y", "K", "V"):
            a, b2 = getattr(dA, name), getattr(dB, name)
            if a.dtype == torch.bfloat16:
                a, b2 = a.view(torch.int16), b2.view(torch.int16)
            np.testing.assert_array_equal(t2n(a), t2n(b2), err_msg="%s differs at step %d" % (name, step))
        np.testing.assert_array_equal(t2n(ecA), t2n(ecB))
        np.testing.assert_array_equal(t2n(eiA)[t2n(ecA) == 1], t2n(eiB)[t2n(ecB) == 1])
        # oracle, free running
        x = np.ascontiguousarray(qn.reshape(g.route_rows, g.d_r))
        idx, gates, _ = orc.route(x, ref.W_r, g.k, bias=ref.bias, dtype=g.dtype)
        np.testing.assert_array_equal(t2n(dA.topk), idx)
        mask = np.zeros((g.B, g.E), np.int32)
        for b in range(g.B):
            mask[b, idx[b]] = 1
        ridx, rcnt = orc.evict(ref.utility, ref.n_valid, g.S - 1, shard_mask=mask, max_evict=1)
        np.testing.assert_array_equal(t2n(ecA), rcnt)
        orc.append(kn, vn, idx, ref.K_shards, ref.V_shards, ref.utility, ref.n_valid, dtype=g.dtype,
                   reuse_idx=ridx, reuse_cnt=rcnt)
        ref.q = qn
        out = oracle_step(ref, idx, gates, orc.COMBINE_LSE, utility=ref.utility, decay=0.9)
        ok, emax, l2 = y_tolerance_ok(t2n(dA.y), out["y"], g.dtype)
        assert ok, (step, emax, l2)
        assert_utility_close(t2n(dA.utility), ref.utility)
        np.testing.assert_array_equal(t2n(dA.n_valid), ref.n_valid)


@pytest.mark.parametrize("bad", ["workspace_alignment", "workspace_size", "nan_scale", "missing_decoder"])
def test_rejected_fused_step_leaves_the_cache_untouched(bad):
    """Argument errors of the attention pass are found before the step's first launch: after a
    rejected call no row, utility, entry count or routing output has changed."""
    from gpu_harness import dev_storage
    spec = dict(B=2, Hq=4, Hkv=4, D=128, E=8, S=64, k=2, dtype="bf16")
    if bad == "missing_decoder":
        spec["rank"] = 32
    g = wl.Geometry(**spec)
    case = wl.make_host_case(g, seed=5, utility0="exp")
    d = DeviceCase(case)
    kn, vn = wl.draw_new_kv(g, 6)
    dkn, dvn = dev_storage(kn, g.dtype), dev_storage(vn, g.dtype)
    ei = torch.full((g.B, g.E, 1), -1, device=DEV, dtype=torch.int32)
    ec = torch.full((g.B, g.E), -5, device=DEV, dtype=torch.int32)
    d.topk.fill_(-7)
    ws, scale, U_K, U_V = d.workspace, 0.0, d.U_K, d.U_V
    if bad == "workspace_alignment":
        big = torch.empty(d.workspace.numel() + 256, device=DEV, dtype=torch.uint8)
        ws = big[16:16 + d.workspace.numel()]
    elif bad == "workspace_size":
        ws = d.workspace[:d.workspace.numel() // 2]
    elif bad == "nan_scale":
        scale = float("nan")
    else:
        U_K = U_V = None
    before = {n: t2n(getattr(d, n).view(torch.int16) if getattr(d, n).dtype == torch.bfloat16 else getattr(d, n))
              for n in ("K", "V", "utility", "n_valid", "topk")}
    with pytest.raises(pk.PikvError) as err:
        pk.pikv_decode_step(d.desc, d.q, d.W_r, d.bias, dkn, dvn, d.K_tab, d.V_tab, U_K, U_V, d.n_valid,
                            d.utility, g.k, pk.COMBINE_LSE, scale, 1.0, d.topk, d.gates, ei, ec, d.y,
                            d.row_max, d.row_norm, d.scores, d.slot_coef, ws)
    assert err.value.status == (-3 if bad == "workspace_size" else -1)
    torch.cuda.synchronize()
    for n, ref in before.items():
        t = getattr(d, n)
        np.testing.assert_array_equal(t2n(t.view(torch.int16) if t.dtype == torch.bfloat16 else t), ref, err_msg=n)
    assert (t2n(ec) == -5).all() and (t2n(ei) == -1).all()


@pytest.mark.gpu
@pytest.mark.parametrize("S", [8, 260, 4096 + 8, 2 * 8192 + 4], ids=lambda S: "S%d" % S)
def test_fused_step_evicts_the_oracles_victim_on_ties_zeros_and_negative_utilities(S):
    """The fused step's scan against the eviction rule on values chosen to separate its cases: every
    shard full; per shard all utilities equal, zeros of both signs, duplicated minima at the ends of
    the threads' ranges, negative values and infinities, ordinary positive ones (S: less than one
    load per thread, a partial pass, one pass and a bit, two passes and a bit)."""
    from gpu_harness import dev_storage
    g = wl.Geometry(B=2, Hq=2, Hkv=2, D=32, E=8, S=S, k=8, dtype="bf16")      # every shard is visited
    case = wl.make_host_case(g, seed=77, utility0="exp")
    rng = np.random.default_rng(S)
    u = np.abs(rng.standard_normal((g.B, g.E, S))).astype(np.float32) + 0.5
    u[0, 0, :] = 0.25                                  # all equal: the highest slot goes
    u[0, 1, ::3] = 0.0
    u[0, 1, 1::6] = -0.0                               # a sign bit, and equal to +0 in the order
    lo = np.float32(0.125)
    u[0, 2, [0, S // 2, S - 1]] = lo                   # the minimum three times
    u[0, 3, :] = rng.standard_normal(S).astype(np.float32)         # negative values
    u[0, 4, S // 3] = -np.inf
    u[0, 5, :] = np.inf
    u[0, 5, S // 2] = 3.0e38
    u[0, 6, [3, 4 % S]] = np.float32(1e-45)            # denormals, adjacent slots of two loads
    u[1, 0, S - 1] = lo
    u[1, 1, 0] = lo
    u[1, 2, :] = 0.0                                   # all zero, as after a run of inserts
    u[1, 3, S - 4:] = lo                               # the last load, all four
    case.utility[:] = u
    case.n_valid[:] = S
    dc = DeviceCase(case)
    ei = torch.full((g.B, g.E, 1), -1, device=DEV, dtype=torch.int32)
    ec = torch.full((g.B, g.E), -5, device=DEV, dtype=torch.int32)
    kn, vn = wl.draw_new_kv(g, 5)
    pk.pikv_decode_step(dc.desc, dc.q, dc.W_r, dc.bias, dev_storage(kn, g.dtype), dev_storage(vn, g.dtype),
                        dc.K_tab, dc.V_tab, dc.U_K, dc.U_V, dc.n_valid, dc.utility, g.k, pk.COMBINE_LSE, 0.0, 1.0,
                        dc.topk, dc.gates, ei, ec, dc.y, dc.row_max, dc.row_norm, dc.scores, dc.slot_coef,
                        dc.workspace)
    ridx, rcnt = orc.evict(u.copy(), np.full((g.B, g.E), S, np.int32), S - 1, max_evict=1)
    assert (rcnt == 1).all()
    np.testing.assert_array_equal(t2n(ec), rcnt)
    np.testing.assert_array_equal(t2n(ei), ridx)
    assert ridx[0, 0, 0] == S - 1 and ridx[0, 2, 0] == S - 1 and ridx[1, 1, 0] == 0 and ridx[1, 2, 0] == S - 1


@pytest.mark.parametrize("seed", range(12))
def test_fused_step_is_bit_identical_to_separate_calls_on_random_geometries(seed):
    """The fused step is defined as the sequence of the separate calls: same bits in every piece of
    state after several steps, on shapes nobody hand-picked (both combine modes, decay, fills)."""
    from gpu_harness import dev_storage
    rng = np.random.default_rng(2000 + seed)
    dtype = str(rng.choice(["bf16", "bf16", "f32"]))
    # (expert counts whose W_r rows are whole aligned 16-byte chunks, and others: the router's
    # generic form inside the step)
    E = int(rng.choice([8, 16, 32, 5, 12, 24, 33] if dtype == "bf16" else [4, 8, 16, 3, 6, 13]))
    D = int(rng.choice([32, 64, 128]))
    rank = int(rng.choice([0, 0, 16, 32]))
    if rank >= D:
        rank = 0
    Hkv = int(rng.choice([1, 2, 4]))
    G = int(rng.choice([1, 2, 3, 4, 8]))
    g = wl.Geometry(B=int(rng.integers(1, 4)), Hq=Hkv * G, Hkv=Hkv, D=D, E=E, S=int(rng.integers(2, 300)),
                    k=int(rng.integers(1, min(E, 6) + 1)), dtype=dtype, rank=rank)
    case = wl.make_host_case(g, seed=seed, utility0="exp", zipf_s=1.1, n_valid=str(rng.choice(["ragged", "full"])))
    combine = int(rng.choice([pk.COMBINE_LSE, pk.COMBINE_LOCAL]))
    decay = float(rng.choice([1.0, 0.9, 0.5]))
    dA, dB = DeviceCase(case), DeviceCase(case)
    eiA = torch.full((g.B, g.E, 1), -1, device=DEV, dtype=torch.int32)
    ecA = torch.full((g.B, g.E), -5, device=DEV, dtype=torch.int32)
    eiB, ecB = eiA.clone(), ecA.clone()
    for step in range(4):
        qn = wl.draw_queries(g, 3000 + 10 * seed + step)
        kn, vn = wl.draw_new_kv(g, 4000 + 10 * seed + step)
        dkn, dvn = dev_storage(kn, g.dtype), dev_storage(vn, g.dtype)
        for d in (dA, dB):
            d.q.copy_(dev_storage(qn, g.dtype))
        pk.pikv_decode_step(dA.desc, dA.q, dA.W_r, dA.bias, dkn, dvn, dA.K_tab, dA.V_tab, dA.U_K, dA.U_V,
                            dA.n_valid, dA.utility, g.k, combine, 0.0, decay, dA.topk, dA.gates,
                            eiA, ecA, dA.y, dA.row_max, dA.row_norm, dA.scores, dA.slot_coef, dA.workspace)
        dB.route()
        pk.pikv_evict(dB.desc, dB.utility, dB.n_valid, g.S - 1, dB.topk, g.k, eiB, ecB, 1, False, None, None)
        pk.pikv_append(dB.desc, dkn, dvn, dB.topk, g.k, eiB, ecB, 1, dB.K_tab, dB.V_tab, dB.utility, dB.n_valid)
        dB.attend(combine=combine)
        dB.update_utility(decay)
        for name in ("topk", "gates", "n_valid", "utility", "y", "row_max", "row_norm", "K", "V"):
            a, b2 = getattr(dA, name), getattr(dB, name)
            if a.dtype == torch.bfloat16:
                a, b2 = a.view(torch.int16), b2.view(torch.int16)
            np.testing.assert_array_equal(t2n(a), t2n(b2), err_msg="%s differs at step %d for %s" % (name, step, g))
        np.testing.assert_array_equal(t2n(ecA), t2n(ecB))
        np.testing.assert_array_equal(t2n(eiA)[t2n(ecA) == 1], t2n(eiB)[t2n(ecB) == 1])


def test_fused_decode_step_without_insert_and_unsupported_shapes():
    g = wl.Geometry(B=2, Hq=4, Hkv=4, D=64, E=8, S=80, k=2, dtype="bf16")
    case = wl.make_host_case(g, seed=42, utility0="exp")
    ensure_route_margin(case, g.k)
    dA, dB = DeviceCase(case), DeviceCase(case)
    pk.pikv_decode_step(dA.desc, dA.q, dA.W_r, dA.bias, None, None, dA.K_tab, dA.V_tab, None, None,
                        dA.n_valid, dA.utility, g.k, pk.COMBINE_LOCAL, 0.0, 1.0, dA.topk, dA.gates,
                        None, None, dA.y, dA.row_max, dA.row_norm, dA.scores, dA.slot_coef, dA.workspace)
    dB.route()
    dB.attend(combine=pk.COMBINE_LOCAL)
    dB.update_utility(1.0)
    for name in ("topk", "y", "utility", "n_valid"):
        np.testing.assert_array_equal(t2n(getattr(dA, name)), t2n(getattr(dB, name)))
    # per-head routing is not served by the fused step
    g2 = wl.Geometry(B=1, Hq=4, Hkv=4, D=64, E=4, S=32, k=2, dtype="f32", per_head_routing=True)
    d2 = DeviceCase(wl.make_host_case(g2, seed=1))
    with pytest.raises(pk.PikvError) as ei:
        pk.pikv_decode_step(d2.desc, d2.q, d2.W_r, None, None, None, d2.K_tab, d2.V_tab, None, None,
                            d2.n_valid, d2.utility, g2.k, pk.COMBINE_LSE, 0.0, 1.0, d2.topk, d2.gates,
                            None, None, d2.y, d2.row_max, d2.row_norm, d2.scores, d2.slot_coef, d2.workspace)
    assert ei.value.status == -2


# ------------------------------------------------ widened rows: router penalties, compress-on-insert
@pytest.mark.parametrize("mode", [0, 1, 2], ids=["load_balance", "cache_aware", "entropy"])
def test_router_penalty_matches_oracle_and_closes_the_loop(mode):
    """Table 1 penalty terms kept on the device: counters exact, bias to fp32 rounding, and the
    penalised routing decisions of a 10-step chain equal the oracle's."""
    from gpu_harness import dev_storage
    g = wl.Geometry(B=6, Hq=4, Hkv=4, D=64, E=8, S=16, k=2, dtype="bf16")
    case = wl.make_host_case(g, seed=51)
    dc = DeviceCase(case)
    rng = np.random.default_rng(3)
    miss_h = rng.integers(0, 50, size=g.E).astype(np.int32)
    load_h = np.zeros(g.E, np.int32)
    load_d = torch.zeros(g.E, device=DEV, dtype=torch.int32)
    miss_d = torch.from_numpy(miss_h).to(DEV)
    bias_d = torch.zeros(g.E, device=DEV)
    dc.bias = bias_d
    coef = (0.05, 0.3, 4.0)[mode]
    bias_h = np.zeros(g.E, np.float32)
    for step in range(10):
        probe = case.clone()
        probe.q = wl.draw_queries(g, 300 + step)
        probe.bias = bias_h
        ensure_route_margin(probe, g.k)
        dc.q.copy_(dev_storage(probe.q, g.dtype))
        dc.route()
        x = np.ascontiguousarray(probe.q.reshape(g.route_rows, g.d_r))
        idx, _, _ = orc.route(x, case.W_r, g.k, bias=bias_h, dtype=g.dtype)
        np.testing.assert_array_equal(t2n(dc.topk), idx)
        pk.pikv_router_penalty(mode, dc.topk, g.route_rows, g.k, g.E, load_d, miss_d, coef, bias_d)
        bias_h = orc.router_penalty(mode, idx, load_h, coef, miss=miss_h)
        np.testing.assert_array_equal(t2n(load_d), load_h)
        np.testing.assert_allclose(t2n(bias_d), bias_h, rtol=1e-5, atol=1e-6)
    assert load_h.sum() == 10 * g.route_rows * g.k


@pytest.mark.parametrize("mode", [0, 1, 2], ids=["load_balance", "cache_aware", "entropy"])
def test_router_feedback_inside_the_fused_step_equals_the_separate_penalty_call(mode):
    """pikv_decode_step_policy with a pikv_router_feedback: the step's last launch updates the
    load counters and the next step's bias exactly as pikv_router_penalty after the step would
    (same bits, every step of a closed loop), and the loop's selections equal the oracle's."""
    from gpu_harness import dev_storage
    g = wl.Geometry(B=5, Hq=8, Hkv=4, D=64, E=8, S=40, k=2, dtype="bf16")
    case = wl.make_host_case(g, seed=52, utility0="exp")
    dA, dB = DeviceCase(case), DeviceCase(case)
    rng = np.random.default_rng(4)
    miss_h = rng.integers(0, 50, size=g.E).astype(np.int32)
    coef = (0.05, 0.3, 4.0)[mode]
    state = {}
    for name, d in (("A", dA), ("B", dB)):
        state[name] = dict(load=torch.zeros(g.E, device=DEV, dtype=torch.int32), miss=torch.from_numpy(miss_h).to(DEV),
                           bias=torch.zeros(g.E, device=DEV),
                           ei=torch.full((g.B, g.E, 1), -1, device=DEV, dtype=torch.int32),
                           ec=torch.zeros((g.B, g.E), device=DEV, dtype=torch.int32))
        d.bias = state[name]["bias"]
    fb = pk.make_router_feedback(mode, coef, state["A"]["load"], state["A"]["bias"], miss=state["A"]["miss"])
    load_h, bias_h = np.zeros(g.E, np.int32), np.zeros(g.E, np.float32)
    for step in range(8):
        probe = case.clone()
        probe.q = wl.draw_queries(g, 400 + step)
        probe.bias = bias_h
        ensure_route_margin(probe, g.k)
        kn, vn = wl.draw_new_kv(g, 450 + step)
        dkn, dvn = dev_storage(kn, g.dtype), dev_storage(vn, g.dtype)
        for d in (dA, dB):
            d.q.copy_(dev_storage(probe.q, g.dtype))
        sA, sB = state["A"], state["B"]
        pk.pikv_decode_step_policy(dA.desc, dA.q, dA.W_r, dA.bias, dkn, dvn, dA.K_tab, dA.V_tab, None, None,
                                   dA.n_valid, dA.utility, g.k, pk.COMBINE_LSE, 0.0, 0.9, dA.topk, dA.gates,
                                   sA["ei"], sA["ec"], dA.y, dA.row_max, dA.row_norm, dA.scores, dA.slot_coef,
                                   dA.workspace, None, feedback=fb)
        pk.pikv_decode_step(dB.desc, dB.q, dB.W_r, dB.bias, dkn, dvn, dB.K_tab, dB.V_tab, None, None,
                            dB.n_valid, dB.utility, g.k, pk.COMBINE_LSE, 0.0, 0.9, dB.topk, dB.gates,
                            sB["ei"], sB["ec"], dB.y, dB.row_max, dB.row_norm, dB.scores, dB.slot_coef,
                            dB.workspace)
        pk.pikv_router_penalty(mode, dB.topk, g.route_rows, g.k, g.E, sB["load"], sB["miss"], coef, sB["bias"])
        for name in ("topk", "y", "utility", "n_valid"):
            np.testing.assert_array_equal(t2n(getattr(dA, name)), t2n(getattr(dB, name)), err_msg=name)
        np.testing.assert_array_equal(t2n(sA["load"]), t2n(sB["load"]))
        np.testing.assert_array_equal(t2n(sA["bias"]).view(np.uint32), t2n(sB["bias"]).view(np.uint32))
        # the oracle's closed loop
        x = np.ascontiguousarray(probe.q.reshape(g.route_rows, g.d_r))
        idx, _, _ = orc.route(x, case.W_r, g.k, bias=bias_h, dtype=g.dtype)
        np.testing.assert_array_equal(t2n(dA.topk), idx)
        bias_h = orc.router_penalty(mode, idx, load_h, coef, miss=miss_h)
        np.testing.assert_array_equal(t2n(sA["load"]), load_h)
        np.testing.assert_allclose(t2n(sA["bias"]), bias_h, rtol=1e-5, atol=1e-6)


@pytest.mark.parametrize("spec", [
    dict(B=3, Hq=4, Hkv=4, D=128, E=4, S=300, k=2, dtype="bf16", rank=32),
    dict(B=2, Hq=8, Hkv=2, D=64, E=4, S=130, k=3, dtype="f32", rank=16),
    dict(B=2, Hq=4, Hkv=4, D=128, E=3, S=200, k=2, dtype="bf16", rank=64),
], ids=["bf16_r32", "f32_r16_gqa4", "bf16_r64"])
@pytest.mark.parametrize("combine", [orc.COMBINE_LSE, orc.COMBINE_LOCAL], ids=["lse", "local"])
def test_value_decoder_bias_matches_oracle(spec, combine):
    """Table 2 row LoRA++ on the value side: U_V carries one more row per kv head, the additive
    term of the decoder; outputs against the oracle's explicit decode with that term, an empty
    selection still gives zero, utilities are those of the run without the term."""
    from gpu_harness import dev_storage
    g = wl.Geometry(**spec)
    case = wl.make_host_case(g, seed=61, n_valid="ragged", utility0="exp")
    case.n_valid[-1, :] = 0                                   # the last sequence: every shard empty
    ensure_route_margin(case, g.k)
    rng = np.random.default_rng(62)
    b_V = wl.encode(rng.standard_normal((g.Hkv, g.D)), g.dtype)
    dc = DeviceCase(case)
    UVb = np.concatenate([case.U_V, b_V[:, None, :]], axis=1)            # [Hkv, rank + 1, D]
    dc.U_V = dev_storage(np.ascontiguousarray(UVb), g.dtype)
    dc.desc = pk.make_desc(g.B, g.Hq, g.Hkv, g.D, g.E, g.S, rank=g.rank,
                           dtype=pk.binding.F32 if g.dtype == "f32" else pk.binding.BF16,
                           stride_h=dc.stride_h, stride_s=dc.stride_s, flags=pk.DESC_VALUE_BIAS)
    dc.route()
    dc.attend(combine=combine)
    dc.update_utility(1.0)
    idx, gates = t2n(dc.topk), t2n(dc.gates)
    u_ref = case.utility.copy()
    ref = orc.attend(case.q, case.K_shards, case.V_shards, case.n_valid, idx, gates, Hkv=g.Hkv, E=g.E, S=g.S,
                     dtype=g.dtype, rank=g.rank, U_K=case.U_K, U_V=case.U_V, V_bias=b_V, combine=combine,
                     utility=u_ref)
    y = t2n(dc.y)
    ok, emax, l2 = y_tolerance_ok(y, ref["y"], g.dtype)
    assert ok, (emax, l2)
    assert (y[-1] == 0).all()
    assert_utility_close(t2n(dc.utility), u_ref)
    # and the difference to the run without the term is the term itself
    plain = DeviceCase(case)
    plain.route()
    plain.attend(combine=combine)
    diff = y[:-1] - t2n(plain.y)[:-1]
    want = wl.decode(b_V, g.dtype)[np.arange(g.Hq) // (g.Hq // g.Hkv)][None]
    np.testing.assert_allclose(diff, np.broadcast_to(want, diff.shape), rtol=1e-5, atol=1e-5)


@pytest.mark.parametrize("spec", [
    dict(B=16, Hq=32, Hkv=32, D=128, E=2, S=8, k=1, dtype="bf16", rank=32),     # config-5 shape
    dict(B=3, Hq=4, Hkv=2, D=64, E=2, S=8, k=1, dtype="bf16", rank=16),
    dict(B=2, Hq=2, Hkv=2, D=128, E=2, S=8, k=1, dtype="f32", rank=64),
], ids=["c5_shape", "rank16", "f32_rank64"])
def test_compress_matches_oracle(spec):
    """codes = W_enc x: fp32 storage to rounding error; bf16 storage equal to the oracle's
    round-to-nearest-even code except where fp32 vs fp64 summation straddles a rounding
    boundary (then exactly one bf16 step away)."""
    from gpu_harness import dev_storage
    g = wl.Geometry(**spec)
    rng = np.random.default_rng(9)
    x = wl.encode(rng.standard_normal((g.B, g.Hkv, g.D)), g.dtype)
    W = wl.encode(rng.standard_normal((g.Hkv, g.rank, g.D)) / np.sqrt(g.D), g.dtype)
    ref = orc.compress(x, W, dtype=g.dtype)
    desc = pk.make_desc(g.B, g.Hq, g.Hkv, g.D, g.E, g.S, rank=g.rank,
                        dtype=pk.binding.F32 if g.dtype == "f32" else pk.binding.BF16)
    out = torch.zeros((g.B, g.Hkv, g.rank), device=DEV,
                      dtype=torch.float32 if g.dtype == "f32" else torch.bfloat16)
    pk.pikv_compress(desc, dev_storage(x, g.dtype), dev_storage(W, g.dtype), out)
    torch.cuda.synchronize()
    got = wl.to_host(out, g.dtype)
    if g.dtype == "f32":
        np.testing.assert_allclose(got, ref, rtol=1e-5, atol=1e-6)
    else:
        same = got == ref
        assert same.mean() > 0.99
        step = np.abs(got.astype(np.int32) - ref.astype(np.int32))
        assert step.max() <= 1                                  # adjacent bf16 bit patterns


def test_compress_then_insert_then_attend_streams_like_the_oracle():
    """Config-5 style step with compress-on-insert: full-width new K/V -> codes -> fused step."""
    from gpu_harness import dev_storage
    g = wl.Geometry(B=3, Hq=4, Hkv=4, D=128, E=8, S=40, k=2, dtype="bf16", rank=32)
    case = wl.make_host_case(g, seed=61, utility0="exp")
    ensure_route_margin(case, g.k)
    rng = np.random.default_rng(5)
    WK = wl.encode(rng.standard_normal((g.Hkv, g.rank, g.D)) / np.sqrt(g.D), "bf16")
    WV = wl.encode(rng.standard_normal((g.Hkv, g.rank, g.D)) / np.sqrt(g.D), "bf16")
    kfull = wl.encode(rng.standard_normal((g.B, g.Hkv, g.D)), "bf16")
    vfull = wl.encode(rng.standard_normal((g.B, g.Hkv, g.D)), "bf16")
    dc = DeviceCase(case)
    kc = torch.zeros((g.B, g.Hkv, g.rank), device=DEV, dtype=torch.bfloat16)
    vc = torch.zeros_like(kc)
    pk.pikv_compress(dc.desc, dev_storage(kfull, "bf16"), dev_storage(WK, "bf16"), kc,
                     dev_storage(vfull, "bf16"), dev_storage(WV, "bf16"), vc)
    np.testing.assert_array_equal(np.abs(wl.to_host(vc, "bf16").astype(np.int32) -
                                         orc.compress(vfull, WV, dtype="bf16").astype(np.int32)) <= 1, True)
    ei = torch.full((g.B, g.E, 1), -1, device=DEV, dtype=torch.int32)
    ec = torch.zeros((g.B, g.E), device=DEV, dtype=torch.int32)
    pk.pikv_decode_step(dc.desc, dc.q, dc.W_r, dc.bias, kc, vc, dc.K_tab, dc.V_tab, dc.U_K, dc.U_V,
                        dc.n_valid, dc.utility, g.k, pk.COMBINE_LSE, 0.0, 1.0, dc.topk, dc.gates, ei, ec,
                        dc.y, dc.row_max, dc.row_norm, dc.scores, dc.slot_coef, dc.workspace)
    torch.cuda.synchronize()
    # oracle on the GPU's own codes (the codes themselves are checked in test_compress_matches_oracle)
    kc_h, vc_h = wl.to_host(kc, "bf16"), wl.to_host(vc, "bf16")
    ref = case.clone()
    x = np.ascontiguousarray(case.q.reshape(g.route_rows, g.d_r))
    idx, gates, _ = orc.route(x, ref.W_r, g.k, dtype=g.dtype)
    np.testing.assert_array_equal(t2n(dc.topk), idx)
    mask = np.zeros((g.B, g.E), np.int32)
    for b in range(g.B):
        mask[b, idx[b]] = 1
    ridx, rcnt = orc.evict(ref.utility, ref.n_valid, g.S - 1, shard_mask=mask, max_evict=1)
    orc.append(kc_h, vc_h, idx, ref.K_shards, ref.V_shards, ref.utility, ref.n_valid, dtype="bf16",
               reuse_idx=ridx, reuse_cnt=rcnt)
    out = oracle_step(ref, idx, gates, orc.COMBINE_LSE, utility=ref.utility, decay=1.0)
    ok, emax, l2 = y_tolerance_ok(t2n(dc.y), out["y"], g.dtype)
    assert ok, (emax, l2)
    assert_utility_close(t2n(dc.utility), ref.utility)
    for s in range(g.B * g.E):
        np.testing.assert_array_equal(dc.shard_host("K", s), ref.K_shards[s])


def test_strided_shards_on_the_matrix_core_kernel_and_the_fused_step():
    """Rows padded to a larger pitch and extra slots per head (stride_s > width, stride_h > S*stride_s)
    through the grouped-query MFMA kernel, both via the separate calls and the fused step."""
    g = wl.Geometry(B=2, Hq=8, Hkv=2, D=128, E=8, S=150, k=2, dtype="bf16")
    case = wl.make_host_case(g, seed=71, n_valid="ragged", utility0="exp")
    case.n_valid[case.n_valid == g.S] = g.S - 1
    ensure_route_margin(case, g.k)
    x = np.ascontiguousarray(case.q.reshape(g.route_rows, g.d_r))
    idx, gates, _ = orc.route(x, case.W_r, g.k, dtype=g.dtype)
    u_ref = case.utility.copy()
    ref = oracle_step(case, idx, gates, orc.COMBINE_LSE, utility=u_ref, decay=0.5)
    for fused in (False, True):
        dc = DeviceCase(case, stride_pad=(16, 7))
        if fused:
            pk.pikv_decode_step(dc.desc, dc.q, dc.W_r, dc.bias, None, None, dc.K_tab, dc.V_tab, None, None,
                                dc.n_valid, dc.utility, g.k, pk.COMBINE_LSE, 0.0, 0.5, dc.topk, dc.gates,
                                None, None, dc.y, dc.row_max, dc.row_norm, dc.scores, dc.slot_coef,
                                dc.workspace)
        else:
            dc.route()
            dc.attend()
            dc.update_utility(0.5)
        np.testing.assert_array_equal(t2n(dc.topk), idx)
        ok, emax, l2 = y_tolerance_ok(t2n(dc.y), ref["y"], g.dtype)
        assert ok, (fused, emax, l2)
        assert_utility_close(t2n(dc.utility), u_ref)


@pytest.mark.parametrize("spec", [
    dict(B=1, Hq=128, Hkv=8, D=128, E=8, S=700, k=4, dtype="bf16"),                    # 16 rows per kv head
    dict(B=2, Hq=256, Hkv=8, D=128, E=8, S=300, k=3, dtype="bf16", tq=8),             # token-major drafts
    dict(B=1, Hq=96, Hkv=96, D=64, E=8, S=120, k=5, dtype="bf16"),                     # plain-ALU kernel
    dict(B=1, Hq=40, Hkv=8, D=32, E=4, S=90, k=2, dtype="f32", rank=16),
], ids=["gqa16_512pairs", "tq8_768pairs", "g1_480pairs", "f32_80pairs"])
@pytest.mark.parametrize("combine", [orc.COMBINE_LSE, orc.COMBINE_LOCAL], ids=["lse", "local"])
def test_fused_step_with_many_head_shard_pairs_equals_separate_calls(spec, combine):
    """More (head, shard) pairs than a utility block has groups of eight lanes: its statistics
    come from one thread per pair, and with many heads per thread the utility blocks are
    dispatched ahead of the merge blocks.  Same bits as the separate calls, two steps in a row."""
    from gpu_harness import dev_storage
    token_major = "tq" in spec
    g = wl.Geometry(token_major=token_major, **spec)
    case = wl.make_host_case(g, seed=77, n_valid="ragged", utility0="exp", w_sigma=0.02)
    ensure_route_margin(case, g.k)
    dA, dB = DeviceCase(case), DeviceCase(case)
    if token_major:
        for d in (dA, dB):
            d.desc = pk.make_desc(g.B, g.Hq, g.Hkv, g.D, g.E, g.S, dtype=pk.binding.BF16, stride_h=d.stride_h,
                                  stride_s=d.stride_s, tq=g.tq)
    eiA = torch.full((g.B, g.E, 1), -1, device=DEV, dtype=torch.int32)
    ecA = torch.full((g.B, g.E), -5, device=DEV, dtype=torch.int32)
    eiB, ecB = eiA.clone(), ecA.clone()
    for step in range(2):
        kn, vn = wl.draw_new_kv(g, 500 + step)
        dkn, dvn = dev_storage(kn, g.dtype), dev_storage(vn, g.dtype)
        pk.pikv_decode_step(dA.desc, dA.q, dA.W_r, dA.bias, dkn, dvn, dA.K_tab, dA.V_tab, dA.U_K, dA.U_V,
                            dA.n_valid, dA.utility, g.k, combine, 0.0, 0.9, dA.topk, dA.gates,
                            eiA, ecA, dA.y, dA.row_max, dA.row_norm, dA.scores, dA.slot_coef, dA.workspace)
        dB.route()
        pk.pikv_evict(dB.desc, dB.utility, dB.n_valid, g.S - 1, dB.topk, g.k, eiB, ecB, 1, False, None, None)
        pk.pikv_append(dB.desc, dkn, dvn, dB.topk, g.k, eiB, ecB, 1, dB.K_tab, dB.V_tab, dB.utility, dB.n_valid)
        dB.attend(combine=combine)
        dB.update_utility(0.9)
        for name in ("topk", "gates", "n_valid", "utility", "y", "row_max", "row_norm", "slot_coef"):
            np.testing.assert_array_equal(t2n(getattr(dA, name)), t2n(getattr(dB, name)),
                                          err_msg="%s differs at step %d" % (name, step))


def test_fused_step_with_many_heads_times_shards_uses_the_separate_merge():
    """Hq * k beyond what a utility block restages: the step falls back to separate merge and
    utility launches and still equals the separate calls bit for bit."""
    g = wl.Geometry(B=1, Hq=64, Hkv=64, D=16, E=64, S=24, k=40, dtype="bf16")
    case = wl.make_host_case(g, seed=72, utility0="exp", w_sigma=0.2)
    ensure_route_margin(case, g.k, margin=1e-4)
    dA, dB = DeviceCase(case), DeviceCase(case)
    pk.pikv_decode_step(dA.desc, dA.q, dA.W_r, dA.bias, None, None, dA.K_tab, dA.V_tab, None, None,
                        dA.n_valid, dA.utility, g.k, pk.COMBINE_LSE, 0.0, 1.0, dA.topk, dA.gates,
                        None, None, dA.y, dA.row_max, dA.row_norm, dA.scores, dA.slot_coef, dA.workspace)
    dB.route()
    dB.attend()
    dB.update_utility(1.0)
    for name in ("topk", "y", "utility"):
        np.testing.assert_array_equal(t2n(getattr(dA, name)), t2n(getattr(dB, name)))
    x = np.ascontiguousarray(case.q.reshape(g.route_rows, g.d_r))
    idx, gates, _ = orc.route(x, case.W_r, g.k, dtype=g.dtype)
    np.testing.assert_array_equal(t2n(dA.topk), idx)
    u_ref = case.utility.copy()
    ref = oracle_step(case, idx, gates, orc.COMBINE_LSE, utility=u_ref)
    ok, emax, l2 = y_tolerance_ok(t2n(dA.y), ref["y"], g.dtype)
    assert ok, (emax, l2)
    assert_utility_close(t2n(dA.utility), u_ref)


# ------------------------------------------------------------------- HIP graph replay
@pytest.mark.parametrize("spec", [
    dict(B=2, Hq=8, Hkv=2, D=128, E=8, S=96, k=2, dtype="bf16"),            # matrix-core kernel
    dict(B=3, Hq=4, Hkv=4, D=64, E=8, S=80, k=3, dtype="bf16", rank=16),   # plain-ALU kernel, codes
], ids=["gqa4_d128", "rank16"])
def test_graph_replays_of_the_fused_step_equal_eager_steps(spec):
    """The benchmark times a captured graph of fused steps.  Every replay must leave exactly the
    state the same number of eager steps leaves (the step carries state: utilities, entry counts,
    evicted rows), with eager work and synchronisations of the program's own between replays."""
    from gpu_harness import dev_storage
    g = wl.Geometry(**spec)
    case = wl.make_host_case(g, seed=101, utility0="exp", zipf_s=1.1)
    kn, vn = wl.draw_new_kv(g, 102)
    per_graph, replays = 3, 4

    def run(dc, ei, ec, dkn, dvn):
        pk.pikv_decode_step(dc.desc, dc.q, dc.W_r, dc.bias, dkn, dvn, dc.K_tab, dc.V_tab, dc.U_K, dc.U_V,
                            dc.n_valid, dc.utility, g.k, pk.COMBINE_LSE, 0.0, 0.9, dc.topk, dc.gates, ei, ec,
                            dc.y, dc.row_max, dc.row_norm, dc.scores, dc.slot_coef, dc.workspace)

    def fresh():
        dc = DeviceCase(case)
        ei = torch.full((g.B, g.E, 1), -1, device=DEV, dtype=torch.int32)
        ec = torch.zeros((g.B, g.E), device=DEV, dtype=torch.int32)
        return dc, ei, ec, dev_storage(kn, g.dtype), dev_storage(vn, g.dtype)

    # eager reference trajectory, a snapshot after every per_graph steps
    dE = fresh()
    snaps = []
    for r in range(replays + 1):                  # +1: the capture pass itself executes nothing, warm-up does
        for _ in range(per_graph):
            run(*dE)
        snaps.append([t2n(x).copy() for x in (dE[0].utility, dE[0].n_valid, dE[0].y, dE[0].topk, dE[2])])

    dG = fresh()
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        for _ in range(per_graph):                # warm-up = the first per_graph steps of the trajectory
            run(*dG)
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            for _ in range(per_graph):
                run(*dG)
        for r in range(replays):
            graph.replay()
            stream.synchronize()
            got = [t2n(x) for x in (dG[0].utility, dG[0].n_valid, dG[0].y, dG[0].topk, dG[2])]
            for a, b2, nm in zip(got, snaps[r + 1], ("utility", "n_valid", "y", "topk", "evicted_cnt")):
                np.testing.assert_array_equal(a, b2, err_msg="%s differs after replay %d" % (nm, r))
            # eager work of the program's own between replays (must not disturb the captured launches)
            scratch = torch.rand(1 << 16, device=DEV)
            assert float((scratch * 2).sum().item()) > 0


@pytest.mark.parametrize("spec", [
    dict(B=1, Hq=4, Hkv=2, D=128, E=3, S=400, k=2, dtype="bf16"),            # matrix-core kernel
    dict(B=2, Hq=2, Hkv=2, D=64, E=3, S=300, k=2, dtype="bf16"),             # plain-ALU kernel
    dict(B=1, Hq=2, Hkv=2, D=64, E=2, S=200, k=2, dtype="f32", rank=16),
], ids=["gqa2_d128", "g1_d64", "f32_rank16"])
def test_attention_with_very_peaked_scores(spec):
    """Scores in the hundreds (scale 8 on N(0,1) data): the softmax is a near one-hot, every
    exponent but a few underflows; nothing may overflow or lose the dominant entry.

    Tolerance: a probability is coef * exp(s - M) with s and M computed in fp32.  A score of
    magnitude |s| carries an absolute error of a few units in its last place (a 128-term fp32 dot
    product times the scale: at most 4 ulp here), so exp(s - M) carries that as a RELATIVE error,
    twice (s and M).  The utility bar of rel 1e-4 therefore widens by 8 ulp32(max |M|) - for
    |M| ~ 300 that is 2.4e-4 - and the row maximum itself is good to 4 ulp32(|M|)."""
    g = wl.Geometry(**spec)
    case = wl.make_host_case(g, seed=23, n_valid="ragged", utility0="exp")
    idx, gates = random_selection(g, 24)
    for combine in (orc.COMBINE_LSE, orc.COMBINE_LOCAL):
        u_ref = case.utility.copy()
        ref = oracle_step(case, idx, gates, combine, utility=u_ref, decay=1.0, scale=8.0)
        dc = DeviceCase(case)
        d_idx, d_gates = torch.from_numpy(idx).to(DEV), torch.from_numpy(gates).to(DEV)
        dc.attend(topk=d_idx, gates=d_gates, combine=combine, scale=8.0)
        dc.update_utility(1.0, topk=d_idx)
        y = t2n(dc.y)
        assert np.isfinite(y).all()
        ok, emax, l2 = y_tolerance_ok(y, ref["y"], g.dtype)
        assert ok, (combine, emax, l2)
        ulp = float(np.spacing(np.float32(np.abs(ref["row_max"][np.isfinite(ref["row_max"])]).max())))
        np.testing.assert_allclose(t2n(dc.row_max), ref["row_max"], rtol=0, atol=4 * ulp)
        u = t2n(dc.utility)
        assert np.isfinite(u).all()
        np.testing.assert_allclose(u, u_ref, rtol=1e-4 + 8 * ulp, atol=1e-9)


def test_stream_read_probe_folds_every_word_once():
    """The measurement kernel behind bench.py's read-ceiling figure reads every byte it is given
    exactly once: its per-span xor of 32-bit words equals numpy's, for spans with ragged ends."""
    rng = np.random.default_rng(3)
    for n, words, parts in ((3, 70000, 5), (1, 4, 1), (2, 1024 * 37 + 12, 7), (4, 16384 * 4, 4)):
        host = rng.integers(0, 2 ** 32, size=(n, words), dtype=np.uint64).astype(np.uint32)
        bufs = [torch.from_numpy(host[i].view(np.int32).copy()).to(DEV) for i in range(n)]
        table = pk.shard_table(bufs)
        out = torch.zeros(n * parts, device=DEV, dtype=torch.int32)
        pk.pikv_stream_read_probe(table, n, words * 4, parts, out)
        got = t2n(out).view(np.uint32).reshape(n, parts)
        span = -(-(words * 4) // parts)
        span = -(-span // 4096) * 4096 // 4
        for i in range(n):
            for pt in range(parts):
                want = np.bitwise_xor.reduce(host[i, pt * span:(pt + 1) * span]) if pt * span < words else 0
                assert got[i, pt] == want, (n, words, parts, i, pt)
