"""Pins of the CPU oracle against things other than itself.

Every check here compares ``oracle/`` with a closed form, a library routine (numpy's
matmul / argsort / sort), a brute force, or an invariant of the definitions in the
paper (Section 3.2 routing mask with exactly k ones; Algorithm 1 attention over the
selected shards only; Table 3 H2O utility = attention mass; eviction under bounded
memory).  They are chosen so that a dropped term, a wrong sign/index or a transposed
operand inside the oracle fails at least one of them.
"""
import numpy as np
import pytest

import workloads as wl
from oracle import pikv_oracle as orc


# ------------------------------------------------------------ independent helpers
def np_softmax(x, axis=-1):
    x = x - x.max(axis=axis, keepdims=True)
    e = np.exp(x)
    return e / e.sum(axis=axis, keepdims=True)


def np_dense_attention(q, K, V, scale):
    """q [D], K [n,D], V [n,D] (float64) -> softmax(q K^T * scale) V, and the weights."""
    p = np_softmax((K @ q) * scale)
    return p @ V, p


def shards_f64(case, which="K"):
    g = case.geo
    src = case.K_shards if which == "K" else case.V_shards
    return [wl.decode(s, g.dtype).astype(np.float64) for s in src]


def run_attend(case, idx, gates, **kw):
    g = case.geo
    return orc.attend(case.q, case.K_shards, case.V_shards, case.n_valid, idx, gates,
                      Hkv=g.Hkv, E=g.E, S=g.S, dtype=g.dtype, rank=g.rank, U_K=case.U_K,
                      U_V=case.U_V, **kw)


def small_geo(**kw):
    base = dict(B=2, Hq=4, Hkv=2, D=16, E=4, S=24, k=2, dtype="f32")
    base.update(kw)
    return wl.Geometry(**base)


# ---------------------------------------------------------------------- route
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_route_logits_are_x_times_W(dtype):
    rng = np.random.default_rng(1)
    x = wl.encode(rng.standard_normal((5, 48)), dtype)
    W = wl.encode(rng.standard_normal((48, 6)), dtype)
    bias = rng.standard_normal(6).astype(np.float32)
    _, _, _, logits = orc.route(x, W, 3, bias=bias, dtype=dtype, want_logits=True)
    ref = wl.decode(x, dtype).astype(np.float64) @ wl.decode(W, dtype).astype(np.float64) + bias
    np.testing.assert_allclose(logits, ref, rtol=1e-12, atol=1e-12)


def test_route_softmax_sums_to_one_and_matches_numpy():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((7, 32)).astype(np.float32)
    W = rng.standard_normal((32, 9)).astype(np.float32)
    idx, gates, probs = orc.route(x, W, 4)
    np.testing.assert_allclose(probs.sum(-1), 1.0, atol=1e-6)
    ref = np_softmax(x.astype(np.float64) @ W.astype(np.float64))
    np.testing.assert_allclose(probs, ref, rtol=1e-6)
    np.testing.assert_allclose(gates.sum(-1), 1.0, atol=1e-6)
    # gates = p renormalised over the selected experts == softmax over selected logits
    sel = np.take_along_axis(ref, idx.astype(np.int64), axis=1)
    np.testing.assert_allclose(gates, sel / sel.sum(-1, keepdims=True), rtol=1e-6)


def test_route_shift_invariance_and_bias_is_additive():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((6, 20)).astype(np.float32)
    W = rng.standard_normal((20, 8)).astype(np.float32)
    i0, g0, p0 = orc.route(x, W, 3)
    i1, g1, p1 = orc.route(x, W, 3, bias=np.full(8, 3.25, np.float32))
    assert (i0 == i1).all()
    np.testing.assert_allclose(g0, g1, rtol=1e-6)
    np.testing.assert_allclose(p0, p1, rtol=1e-6)
    # a large penalty on the winner removes it from the mask
    bias = np.zeros(8, np.float32)
    bias[i0[0, 0]] = -100.0
    i2, _, _ = orc.route(x[:1].copy(), W, 3, bias=bias)
    assert i0[0, 0] not in i2[0]


def test_route_k_equals_E_is_argsort_and_k1_gate_is_one():
    rng = np.random.default_rng(4)
    x = rng.standard_normal((9, 16)).astype(np.float32)
    W = rng.standard_normal((16, 5)).astype(np.float32)
    logits = x.astype(np.float64) @ W.astype(np.float64)
    idx, gates, probs = orc.route(x, W, 5)
    assert (idx == np.argsort(-logits, axis=1, kind="stable")).all()
    np.testing.assert_allclose(gates, np.take_along_axis(probs, idx.astype(np.int64), 1), rtol=1e-6)
    idx1, gates1, _ = orc.route(x, W, 1)
    assert (idx1[:, 0] == logits.argmax(1)).all()
    np.testing.assert_array_equal(gates1, np.ones_like(gates1))


def test_route_two_experts_closed_form_sigmoid():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((11, 12)).astype(np.float32)
    W = rng.standard_normal((12, 2)).astype(np.float32)
    logits = x.astype(np.float64) @ W.astype(np.float64)
    _, _, probs = orc.route(x, W, 1)
    sig = 1.0 / (1.0 + np.exp(-(logits[:, 0] - logits[:, 1])))
    np.testing.assert_allclose(probs[:, 0], sig, rtol=1e-6)


def test_route_topk_equals_brute_force_with_exact_ties():
    # integer-valued inputs: logits are exact, duplicate columns create exact ties;
    # the mask must hold exactly k distinct experts, lower index first among equals.
    rng = np.random.default_rng(6)
    x = rng.integers(-3, 4, size=(40, 10)).astype(np.float32)
    Wb = rng.integers(-2, 3, size=(10, 4)).astype(np.float32)
    W = np.concatenate([Wb, Wb[:, [1, 3]], Wb[:, [0]]], axis=1)        # E = 7, ties
    logits = (x.astype(np.int64) @ W.astype(np.int64))
    for k in (1, 2, 3, 5, 7):
        idx, gates, _ = orc.route(x, W, k)
        for r in range(x.shape[0]):
            order = sorted(range(7), key=lambda e: (-logits[r, e], e))[:k]
            assert list(idx[r]) == order
            assert len(set(idx[r])) == k
    # the all-equal row: experts 0..k-1 in index order, uniform gates
    idx, gates, probs = orc.route(np.zeros((1, 10), np.float32), W, 3)
    assert list(idx[0]) == [0, 1, 2]
    np.testing.assert_allclose(gates[0], 1 / 3, rtol=1e-6)
    np.testing.assert_allclose(probs[0], 1 / 7, rtol=1e-6)


# ------------------------------------------------------------------ attention
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("nv", ["full", "ragged"])
def test_k_equals_E_without_gates_is_dense_attention(dtype, nv):
    """Mask of all ones: attention over C[g] is attention over the whole cache."""
    g = small_geo(dtype=dtype, k=4)
    case = wl.make_host_case(g, seed=7, n_valid=nv)
    perm = np.stack([np.random.default_rng(8 + b).permutation(g.E) for b in range(g.B)]).astype(np.int32)
    out = run_attend(case, perm, None, want_prob=True)
    Kf, Vf = shards_f64(case, "K"), shards_f64(case, "V")
    qf = wl.decode(case.q, dtype).astype(np.float64)
    scale = 1.0 / np.sqrt(g.D)
    for b in range(g.B):
        for h in range(g.Hq):
            hk = h // g.G
            Kc = np.concatenate([Kf[b * g.E + e][hk, :case.n_valid[b, e]] for e in perm[b]])
            Vc = np.concatenate([Vf[b * g.E + e][hk, :case.n_valid[b, e]] for e in perm[b]])
            yref, pref = np_dense_attention(qf[b, h], Kc, Vc, scale)
            np.testing.assert_allclose(out["y"][b, h], yref, rtol=2e-6, atol=1e-7)
            pcat = np.concatenate([out["prob"][b, h, j, :case.n_valid[b, e]]
                                   for j, e in enumerate(perm[b])])
            np.testing.assert_allclose(pcat, pref, rtol=1e-10, atol=1e-15)
            # row_max / row_norm are the joint softmax's max and normaliser
            s = (Kc @ qf[b, h]) * scale
            np.testing.assert_allclose(out["row_max"][b, h], s.max(), rtol=1e-6)
            np.testing.assert_allclose(out["row_norm"][b, h], np.exp(s - s.max()).sum(), rtol=1e-6)


def test_uniform_gates_and_selection_order_do_not_change_lse_result():
    g = small_geo(k=3)
    case = wl.make_host_case(g, seed=9, n_valid="ragged")
    idx = np.array([[2, 0, 3], [1, 3, 0]], np.int32)
    y0 = run_attend(case, idx, None)["y"]
    y1 = run_attend(case, idx, np.full((2, 3), 0.37, np.float32))["y"]
    y2 = run_attend(case, np.ascontiguousarray(idx[:, ::-1]), None)["y"]
    np.testing.assert_allclose(y0, y1, rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(y0, y2, rtol=1e-6, atol=1e-7)


def test_routed_subset_is_dense_attention_over_that_subset_with_gates_as_weights():
    """LSE mode with gates: entry weights are g_e * exp(s_i), normalised jointly."""
    g = small_geo(k=2, B=1)
    case = wl.make_host_case(g, seed=10)
    idx = np.array([[3, 1]], np.int32)
    gates = np.array([[0.8, 0.2]], np.float32)
    out = run_attend(case, idx, gates)
    Kf, Vf = shards_f64(case, "K"), shards_f64(case, "V")
    qf = case.q.astype(np.float64)
    for h in range(g.Hq):
        hk = h // g.G
        Kc = np.concatenate([Kf[e][hk] for e in idx[0]])
        Vc = np.concatenate([Vf[e][hk] for e in idx[0]])
        w = np.exp((Kc @ qf[0, h]) / np.sqrt(g.D)) * np.repeat(gates[0].astype(np.float64), g.S)
        np.testing.assert_allclose(out["y"][0, h], (w / w.sum()) @ Vc, rtol=2e-6, atol=1e-7)


def test_local_mode_k1_is_plain_attention_over_one_shard():
    g = small_geo(k=1)
    case = wl.make_host_case(g, seed=11, n_valid="ragged")
    case.n_valid[case.n_valid == 0] = 5
    idx = np.array([[2], [0]], np.int32)
    for gates in (None, np.array([[0.3], [0.9]], np.float32)):
        out = run_attend(case, idx, gates, combine=orc.COMBINE_LOCAL)
        Kf, Vf = shards_f64(case, "K"), shards_f64(case, "V")
        qf = case.q.astype(np.float64)
        for b in range(g.B):
            e = idx[b, 0]
            n = case.n_valid[b, e]
            for h in range(g.Hq):
                yref, _ = np_dense_attention(qf[b, h], Kf[b * g.E + e][h // g.G, :n],
                                             Vf[b * g.E + e][h // g.G, :n], 1 / np.sqrt(g.D))
                np.testing.assert_allclose(out["y"][b, h], yref, rtol=2e-6, atol=1e-7)


def test_local_mode_is_gate_weighted_sum_of_per_shard_attention():
    g = small_geo(k=3, B=1)
    case = wl.make_host_case(g, seed=12)
    idx = np.array([[0, 2, 3]], np.int32)
    gates = np.array([[0.5, 0.3, 0.1]], np.float32)          # not normalised on purpose
    out = run_attend(case, idx, gates, combine=orc.COMBINE_LOCAL, want_prob=True)
    Kf, Vf = shards_f64(case, "K"), shards_f64(case, "V")
    qf = case.q.astype(np.float64)
    gh = gates[0].astype(np.float64) / gates[0].astype(np.float64).sum()
    for h in range(g.Hq):
        acc = np.zeros(g.D)
        for j, e in enumerate(idx[0]):
            yj, pj = np_dense_attention(qf[0, h], Kf[e][h // g.G], Vf[e][h // g.G], 1 / np.sqrt(g.D))
            acc += gh[j] * yj
            np.testing.assert_allclose(out["prob"][0, h, j], gh[j] * pj, rtol=1e-10)
        np.testing.assert_allclose(out["y"][0, h], acc, rtol=2e-6, atol=1e-7)
    np.testing.assert_allclose(out["row_norm"][0], gates[0].sum(), rtol=1e-6)


def test_local_mode_with_lse_weights_reproduces_dense():
    """Feeding g_e = Z_e e^{m_e} (each shard's softmax mass) to LOCAL gives dense attention."""
    g = small_geo(k=4, B=1)
    case = wl.make_host_case(g, seed=13)
    idx = np.array([[0, 1, 2, 3]], np.int32)
    dense = run_attend(case, idx, None)["y"]
    Kf = shards_f64(case, "K")
    qf = case.q.astype(np.float64)
    # per-head weights differ, so run head by head with Hq = Hkv = 1 slices
    for h in range(g.Hq):
        hk = h // g.G
        mass = np.array([np.exp((Kf[e][hk] @ qf[0, h]) / np.sqrt(g.D)).sum() for e in range(4)])
        sub = wl.Geometry(B=1, Hq=1, Hkv=1, D=g.D, E=4, S=g.S, k=4, dtype="f32")
        Ks = [np.ascontiguousarray(s[hk:hk + 1]) for s in case.K_shards]
        Vs = [np.ascontiguousarray(s[hk:hk + 1]) for s in case.V_shards]
        y = orc.attend(np.ascontiguousarray(case.q[:, h:h + 1]), Ks, Vs, case.n_valid, idx,
                       mass.astype(np.float32)[None], Hkv=1, E=4, S=sub.S,
                       combine=orc.COMBINE_LOCAL)["y"]
        np.testing.assert_allclose(y[0, 0], dense[0, h], rtol=1e-5, atol=1e-6)


@pytest.mark.parametrize("combine", [orc.COMBINE_LSE, orc.COMBINE_LOCAL])
def test_probabilities_sum_to_one_constant_V_and_zero_q(combine):
    g = small_geo(k=2)
    case = wl.make_host_case(g, seed=14, n_valid="ragged")
    case.n_valid[:, 1] = 7
    idx = np.array([[1, 3], [2, 1]], np.int32)
    gates = np.array([[0.6, 0.4], [0.25, 0.75]], np.float32)
    out = run_attend(case, idx, gates, combine=combine, want_prob=True)
    np.testing.assert_allclose(out["prob"].sum(axis=(2, 3)), 1.0, rtol=1e-12)
    # y == sum_i p_i V_i
    Vf = shards_f64(case, "V")
    for b in range(g.B):
        for h in range(g.Hq):
            acc = sum(out["prob"][b, h, j] @ Vf[b * g.E + e][h // g.G] for j, e in enumerate(idx[b]))
            np.testing.assert_allclose(out["y"][b, h], acc, rtol=2e-6, atol=1e-7)
    # constant V rows => y is that row
    c = case.clone()
    const = np.linspace(-1, 1, g.D).astype(np.float32)
    for s in c.V_shards:
        s[:] = const
    np.testing.assert_allclose(run_attend(c, idx, gates, combine=combine)["y"],
                               np.broadcast_to(const, (g.B, g.Hq, g.D)), rtol=1e-6, atol=1e-7)
    # q = 0 => every score is 0: LSE weights g_e per entry; LOCAL weights g_e/n_e per entry
    c = case.clone()
    c.q[:] = 0
    y = run_attend(c, idx, gates, combine=combine)["y"]
    for b in range(g.B):
        for h in range(g.Hq):
            num, den = np.zeros(g.D), 0.0
            for j, e in enumerate(idx[b]):
                n = c.n_valid[b, e]
                if n == 0:
                    continue
                Vm = Vf[b * g.E + e][h // g.G, :n]
                if combine == orc.COMBINE_LSE:
                    num += gates[b, j] * Vm.sum(0)
                    den += gates[b, j] * n
                else:
                    num += gates[b, j] * Vm.mean(0)
                    den += gates[b, j]
            np.testing.assert_allclose(y[b, h], num / den, rtol=2e-6, atol=1e-7)


def test_scale_argument_and_default():
    g = small_geo(k=2, B=1)
    case = wl.make_host_case(g, seed=15)
    idx = np.array([[0, 1]], np.int32)
    y_def = run_attend(case, idx, None)["y"]
    y_exp = run_attend(case, idx, None, scale=1 / np.sqrt(g.D))["y"]
    np.testing.assert_allclose(y_def, y_exp, rtol=1e-6, atol=1e-7)
    y_one = run_attend(case, idx, None, scale=1.0)["y"]
    Kf, Vf = shards_f64(case, "K"), shards_f64(case, "V")
    Kc = np.concatenate([Kf[0][0], Kf[1][0]])
    Vc = np.concatenate([Vf[0][0], Vf[1][0]])
    yref, _ = np_dense_attention(case.q[0, 0].astype(np.float64), Kc, Vc, 1.0)
    np.testing.assert_allclose(y_one[0, 0], yref, rtol=2e-6, atol=1e-7)


def test_gqa_equals_replicated_kv_heads():
    g = small_geo(Hq=6, Hkv=2, k=2)
    case = wl.make_host_case(g, seed=16, n_valid="ragged")
    idx = np.array([[0, 2], [3, 1]], np.int32)
    gates = np.array([[0.7, 0.3], [0.5, 0.5]], np.float32)
    y = run_attend(case, idx, gates)["y"]
    Krep = [np.ascontiguousarray(np.repeat(s, g.G, axis=0)) for s in case.K_shards]
    Vrep = [np.ascontiguousarray(np.repeat(s, g.G, axis=0)) for s in case.V_shards]
    y2 = orc.attend(case.q, Krep, Vrep, case.n_valid, idx, gates, Hkv=g.Hq, E=g.E, S=g.S)["y"]
    np.testing.assert_array_equal(y, y2)
    # and heads of one group really differ from each other / from the other group
    assert not np.allclose(y[:, 0], y[:, 1]) and not np.allclose(y[:, 0], y[:, 3])


def test_per_head_routing_uses_each_heads_own_selection():
    g = small_geo(B=1, Hq=3, Hkv=3, k=1, per_head_routing=True)
    case = wl.make_host_case(g, seed=17)
    idx = np.array([[0], [2], [3]], np.int32)                 # rows = (b, h)
    y = run_attend(case, idx, None)["y"]
    Kf, Vf = shards_f64(case, "K"), shards_f64(case, "V")
    for h in range(3):
        yref, _ = np_dense_attention(case.q[0, h].astype(np.float64), Kf[idx[h, 0]][h],
                                     Vf[idx[h, 0]][h], 1 / np.sqrt(g.D))
        np.testing.assert_allclose(y[0, h], yref, rtol=2e-6, atol=1e-7)


def test_strided_shard_layout():
    """stride_h / stride_s address rows inside a larger buffer."""
    g = small_geo(B=1, k=2)
    case = wl.make_host_case(g, seed=18)
    idx = np.array([[1, 2]], np.int32)
    y = run_attend(case, idx, None)["y"]
    pad_s, pad_h = g.D + 8, (g.S + 3) * (g.D + 8)
    Kp, Vp = [], []
    for Ks, Vs in zip(case.K_shards, case.V_shards):
        kb = np.full((g.Hkv, g.S + 3, g.D + 8), 99.0, np.float32)
        vb = np.full((g.Hkv, g.S + 3, g.D + 8), -99.0, np.float32)
        kb[:, :g.S, :g.D] = Ks
        vb[:, :g.S, :g.D] = Vs
        Kp.append(kb)
        Vp.append(vb)
    y2 = orc.attend(case.q, Kp, Vp, case.n_valid, idx, None, Hkv=g.Hkv, E=g.E, S=g.S,
                    stride_h=pad_h, stride_s=pad_s)["y"]
    np.testing.assert_array_equal(y, y2)


def test_empty_selected_shards():
    g = small_geo(k=2)
    case = wl.make_host_case(g, seed=19)
    case.n_valid[0, :] = 0                    # sequence 0: everything empty
    case.n_valid[1, 2] = 0                    # sequence 1: one of the two selected is empty
    idx = np.array([[0, 1], [2, 3]], np.int32)
    gates = np.array([[0.5, 0.5], [0.9, 0.1]], np.float32)
    for combine in (orc.COMBINE_LSE, orc.COMBINE_LOCAL):
        u = np.ones((g.B, g.E, g.S), np.float32)
        out = orc.attend(case.q, case.K_shards, case.V_shards, case.n_valid, idx, gates,
                         Hkv=g.Hkv, E=g.E, S=g.S, combine=combine, utility=u, decay=0.5,
                         want_prob=True)
        assert (out["y"][0] == 0).all() and (out["prob"][0] == 0).all()
        assert (u[0] == 1).all()                            # nothing visited => untouched
        Kf, Vf = shards_f64(case, "K"), shards_f64(case, "V")
        for h in range(g.Hq):
            yref, _ = np_dense_attention(case.q[1, h].astype(np.float64), Kf[g.E + 3][h // g.G],
                                         Vf[g.E + 3][h // g.G], 1 / np.sqrt(g.D))
            np.testing.assert_allclose(out["y"][1, h], yref, rtol=2e-6, atol=1e-7)


# -------------------------------------------------------------------- low rank
def lowrank_case(seed, rank, D=16, dtype="f32", **kw):
    g = small_geo(D=D, rank=rank, dtype=dtype, **kw)
    return wl.make_host_case(g, seed=seed)


def test_lowrank_identity_decoder_is_bitwise_the_dense_path():
    case = lowrank_case(20, rank=16)
    g = case.geo
    eye = np.broadcast_to(np.eye(16, dtype=np.float32), (g.Hkv, 16, 16)).copy()
    case.U_K, case.U_V = eye, eye.copy()
    idx = np.array([[0, 3], [2, 1]], np.int32)
    y_lr = run_attend(case, idx, None)["y"]
    y_dense = orc.attend(case.q, case.K_shards, case.V_shards, case.n_valid, idx, None,
                         Hkv=g.Hkv, E=g.E, S=g.S)["y"]
    np.testing.assert_array_equal(y_lr, y_dense)


def test_lowrank_crop_decoder_equals_zero_padded_dense():
    """Table 2 'crop to r': decoder [I_r 0] == dense attention on zero-padded rows."""
    case = lowrank_case(21, rank=6)
    g = case.geo
    U = np.zeros((g.Hkv, 6, 16), np.float32)
    U[:, np.arange(6), np.arange(6)] = 1
    case.U_K, case.U_V = U, U.copy()
    idx = np.array([[1, 2], [0, 3]], np.int32)
    gates = np.array([[0.6, 0.4], [0.1, 0.9]], np.float32)
    y_lr = run_attend(case, idx, gates)["y"]
    Kp = [np.ascontiguousarray(np.pad(s, ((0, 0), (0, 0), (0, 10)))) for s in case.K_shards]
    Vp = [np.ascontiguousarray(np.pad(s, ((0, 0), (0, 0), (0, 10)))) for s in case.V_shards]
    y_d = orc.attend(case.q, Kp, Vp, case.n_valid, idx, gates, Hkv=g.Hkv, E=g.E, S=g.S)["y"]
    np.testing.assert_allclose(y_lr, y_d, rtol=1e-6, atol=1e-7)
    assert (y_lr[..., 6:] == 0).all()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_lowrank_explicit_decode_equals_absorbed_projection(dtype):
    """s_i = (U_K q).c_i and y = (sum p_i c_i) U_V, written independently in numpy."""
    case = lowrank_case(22, rank=4, dtype=dtype, B=1, k=2)
    g = case.geo
    idx = np.array([[3, 0]], np.int32)
    out = run_attend(case, idx, None)
    qf = wl.decode(case.q, dtype).astype(np.float64)
    UK = wl.decode(case.U_K, dtype).astype(np.float64)
    UV = wl.decode(case.U_V, dtype).astype(np.float64)
    Kc, Vc = shards_f64(case, "K"), shards_f64(case, "V")
    for h in range(g.Hq):
        hk = h // g.G
        qt = UK[hk] @ qf[0, h]                                   # [r]
        codes_k = np.concatenate([Kc[e][hk] for e in idx[0]])
        codes_v = np.concatenate([Vc[e][hk] for e in idx[0]])
        p = np_softmax((codes_k @ qt) / np.sqrt(g.D))
        np.testing.assert_allclose(out["y"][0, h], (p @ codes_v) @ UV[hk], rtol=3e-6, atol=1e-7)


# --------------------------------------------------------------------- utility
def test_utility_is_accumulated_attention_mass():
    """Table 3 (H2O): decay 1 from zero => total utility == number of (step, head) reads."""
    g = small_geo(k=2)
    case = wl.make_host_case(g, seed=23, n_valid="ragged")
    case.n_valid[case.n_valid == 0] = 3
    u = np.zeros((g.B, g.E, g.S), np.float32)
    steps = 5
    visited = np.zeros((g.B, g.E), bool)
    for t in range(steps):
        case.q = wl.draw_queries(g, 100 + t)
        idx = np.stack([np.random.default_rng(50 + 7 * t + b).permutation(g.E)[:2]
                        for b in range(g.B)]).astype(np.int32)
        for b in range(g.B):
            visited[b, idx[b]] = True
        before = u.copy()
        out = run_attend(case, idx, None, utility=u, want_prob=True)
        # increment equals the head-sum of the returned probabilities
        for b in range(g.B):
            for j, e in enumerate(idx[b]):
                np.testing.assert_allclose(u[b, e] - before[b, e], out["prob"][b, :, j].sum(0),
                                           rtol=1e-5, atol=1e-7)
    np.testing.assert_allclose(u.sum(axis=(1, 2)), steps * g.Hq, rtol=1e-5)
    assert (u >= 0).all() and (u[~visited] == 0).all()
    for b in range(g.B):
        for e in range(g.E):
            assert (u[b, e, case.n_valid[b, e]:] == 0).all()


def test_utility_decay_touches_only_visited_shards():
    g = small_geo(k=1)
    case = wl.make_host_case(g, seed=24)
    u0 = np.random.default_rng(0).random((g.B, g.E, g.S)).astype(np.float32)
    u = u0.copy()
    idx = np.array([[2], [0]], np.int32)
    out = run_attend(case, idx, None, utility=u, decay=0.9, want_prob=True)
    for b in range(g.B):
        for e in range(g.E):
            if e == idx[b, 0]:
                ref = 0.9 * u0[b, e].astype(np.float64) + out["prob"][b, :, 0].sum(0)
                np.testing.assert_allclose(u[b, e], ref, rtol=1e-6)
            else:
                np.testing.assert_array_equal(u[b, e], u0[b, e])


def test_utility_single_entry_shard_gets_exactly_its_gate_share_per_head():
    g = small_geo(k=2, B=1)
    case = wl.make_host_case(g, seed=25)
    case.n_valid[0, 1] = 1
    idx = np.array([[1, 3]], np.int32)
    gates = np.array([[0.25, 0.75]], np.float32)
    u = np.zeros((1, g.E, g.S), np.float32)
    run_attend(case, idx, gates, combine=orc.COMBINE_LOCAL, utility=u)
    np.testing.assert_allclose(u[0, 1, 0], g.Hq * 0.25, rtol=1e-6)
    np.testing.assert_allclose(u[0, 3].sum(), g.Hq * 0.75, rtol=1e-6)


def test_utility_per_head_routing_sums_only_heads_that_selected_the_shard():
    g = small_geo(B=1, Hq=3, Hkv=3, k=1, per_head_routing=True)
    case = wl.make_host_case(g, seed=26)
    idx = np.array([[2], [2], [0]], np.int32)
    u = np.zeros((1, g.E, g.S), np.float32)
    run_attend(case, idx, None, utility=u)
    np.testing.assert_allclose(u[0].sum(-1), [1, 0, 2, 0], rtol=1e-6, atol=1e-7)


# ----------------------------------------------------------------------- evict
def brute_evict(u, n, capacity):
    order = sorted(range(n), key=lambda i: (-float(u[i]), i))
    return sorted(order[capacity:])


@pytest.mark.parametrize("seed", range(4))
def test_evict_equals_brute_force_sort(seed):
    rng = np.random.default_rng(seed)
    B, E, S = 2, 3, 16
    u = rng.integers(0, 5, size=(B, E, S)).astype(np.float32) / 4        # many exact ties
    n = rng.integers(0, S + 1, size=(B, E)).astype(np.int32)
    cap = 6
    u_in, n_in = u.copy(), n.copy()
    idx, cnt = orc.evict(u, n, cap)
    for b in range(B):
        for e in range(E):
            ref = brute_evict(u_in[b, e], n_in[b, e], cap) if n_in[b, e] > cap else []
            assert cnt[b, e] == len(ref)
            assert list(idx[b, e, :cnt[b, e]]) == ref
            assert n[b, e] == min(n_in[b, e], cap)
    np.testing.assert_array_equal(u, u_in)                                # no compaction asked


def test_evict_special_cases():
    S = 10
    u = np.full((1, 1, S), 0.5, np.float32)
    n = np.array([[S]], np.int32)
    idx, cnt = orc.evict(u.copy(), n.copy(), 7)
    assert list(idx[0, 0, :3]) == [7, 8, 9] and cnt[0, 0] == 3           # all equal: highest slots go
    idx, cnt = orc.evict(u.copy(), n.copy(), S)
    assert cnt[0, 0] == 0                                                # capacity >= n: no-op
    n2 = n.copy()
    idx, cnt = orc.evict(u.copy(), n2, 0)
    assert list(idx[0, 0]) == list(range(S)) and n2[0, 0] == 0           # capacity 0: all evicted
    u3 = np.arange(S, dtype=np.float32)[None, None].copy()
    idx, cnt = orc.evict(u3, n.copy(), S - 1)
    assert cnt[0, 0] == 1 and idx[0, 0, 0] == 0                          # evict-1 == argmin
    # mask: unselected shards untouched
    u4 = np.tile(np.arange(S, dtype=np.float32), (1, 2, 1))
    n4 = np.array([[S, S]], np.int32)
    idx, cnt = orc.evict(u4, n4, 4, shard_mask=np.array([[0, 1]], np.int32))
    assert list(cnt[0]) == [0, 6] and list(n4[0]) == [S, 4]


def test_evict_compaction_keeps_order_and_rows():
    rng = np.random.default_rng(5)
    B, E, S, Hkv, w = 1, 2, 12, 2, 4
    u = rng.random((B, E, S)).astype(np.float32)
    n = np.array([[12, 9]], np.int32)
    K = [rng.standard_normal((Hkv, S, w)).astype(np.float32) for _ in range(2)]
    V = [rng.standard_normal((Hkv, S, w)).astype(np.float32) for _ in range(2)]
    u0, K0, V0 = u.copy(), [x.copy() for x in K], [x.copy() for x in V]
    idx, cnt = orc.evict(u, n, 5, compact=True, K_shards=K, V_shards=V, Hkv=Hkv, width=w)
    for e in range(2):
        gone = set(idx[0, e, :cnt[0, e]])
        kept = [i for i in range([12, 9][e]) if i not in gone]
        assert len(kept) == 5 and n[0, e] == 5
        assert sorted(gone) == brute_evict(u0[0, e], [12, 9][e], 5)
        np.testing.assert_array_equal(u[0, e, :5], u0[0, e, kept])
        np.testing.assert_array_equal(K[e][:, :5], K0[e][:, kept])
        np.testing.assert_array_equal(V[e][:, :5], V0[e][:, kept])


# ---------------------------------------------------------------------- append
def test_append_writes_rows_zeroes_utility_and_grows_n():
    g = small_geo(B=2, k=2, dtype="bf16")
    case = wl.make_host_case(g, seed=27, n_valid="ragged", utility0="exp")
    case.n_valid[case.n_valid == g.S] = g.S - 1
    kn, vn = wl.draw_new_kv(g, 3)
    idx = np.array([[0, 2], [3, 1]], np.int32)
    n0 = case.n_valid.copy()
    K0 = [s.copy() for s in case.K_shards]
    orc.append(kn, vn, idx, case.K_shards, case.V_shards, case.utility, case.n_valid, dtype="bf16")
    for b in range(2):
        for e in range(g.E):
            s = b * g.E + e
            if e in idx[b]:
                slot = n0[b, e]
                assert case.n_valid[b, e] == slot + 1
                np.testing.assert_array_equal(case.K_shards[s][:, slot], kn[b])
                np.testing.assert_array_equal(case.V_shards[s][:, slot], vn[b])
                assert case.utility[b, e, slot] == 0
                np.testing.assert_array_equal(case.K_shards[s][:, :slot], K0[s][:, :slot])
            else:
                assert case.n_valid[b, e] == n0[b, e]
                np.testing.assert_array_equal(case.K_shards[s], K0[s])


def test_streaming_step_reuses_the_evicted_slot_and_conserves_counts():
    """Full shard: evict the minimum-utility entry, insert the new entry in its place."""
    g = small_geo(B=2, k=2, S=8)
    case = wl.make_host_case(g, seed=28, utility0="exp")
    idx = np.array([[1, 3], [0, 1]], np.int32)
    mask = np.zeros((g.B, g.E), np.int32)
    for b in range(g.B):
        mask[b, idx[b]] = 1
    u0 = case.utility.copy()
    K0 = [s.copy() for s in case.K_shards]
    eidx, ecnt = orc.evict(case.utility, case.n_valid, g.S - 1, shard_mask=mask, max_evict=1)
    kn, vn = wl.draw_new_kv(g, 4)
    orc.append(kn, vn, idx, case.K_shards, case.V_shards, case.utility, case.n_valid,
               reuse_idx=eidx, reuse_cnt=ecnt)
    assert (case.n_valid == g.S).all()
    for b in range(g.B):
        for e in range(g.E):
            s = b * g.E + e
            changed = [i for i in range(g.S) if not np.array_equal(case.K_shards[s][:, i], K0[s][:, i])]
            if mask[b, e]:
                victim = int(np.argmin(u0[b, e]))
                assert changed == [victim] and eidx[b, e, 0] == victim
                assert case.utility[b, e, victim] == 0
            else:
                assert changed == []


# ------------------------------------------------------------ router penalties
def test_load_balance_penalty_closed_forms():
    """Table 1 row LB: -alpha (mu_e - mean): sums to zero, vanishes for uniform load."""
    load = np.zeros(4, np.int32)
    idx = np.array([[0, 1], [0, 2], [0, 3]], np.int32)
    bias = orc.router_penalty(orc.LB, idx, load, 0.5)
    assert list(load) == [3, 1, 1, 1]
    np.testing.assert_allclose(bias, -0.5 * (np.array([3, 1, 1, 1]) - 1.5), rtol=1e-7)
    assert abs(bias.sum()) < 1e-6
    # counters accumulate over calls; a second, balancing call makes the penalty vanish
    bias = orc.router_penalty(orc.LB, np.array([[1, 2], [3, 1], [2, 3]], np.int32), load, 0.5)
    assert list(load) == [3, 3, 3, 3] and (bias == 0).all()
    # the over-used expert is pushed down, the others up, by amounts proportional to alpha
    b1 = orc.router_penalty(orc.LB, idx, np.zeros(4, np.int32), 1.0)
    b2 = orc.router_penalty(orc.LB, idx, np.zeros(4, np.int32), 2.0)
    assert b1[0] < 0 < b1[1] and np.allclose(b2, 2 * b1)


def test_cache_aware_penalty_is_minus_lambda_log1p_miss():
    miss = np.array([0, 1, 9, 99], np.int32)
    load = np.zeros(4, np.int32)
    bias = orc.router_penalty(orc.CACHE_AWARE, np.array([[2, 3]], np.int32), load, 0.7, miss=miss)
    np.testing.assert_allclose(bias, -0.7 * np.log1p(miss.astype(np.float64)), rtol=1e-6)
    assert bias[0] == 0 and list(load) == [0, 0, 1, 1]


def test_entropy_penalty_closed_forms():
    """Table 1 row E, -beta H(p_e) with p_e the running selection share and H(p_e) = -p_e ln p_e,
    centred over the experts: zero under uniform load, zero-sum, an expert with a larger share
    (all shares below 1/e) is pushed down, linear in beta, and equal to the formula written
    with scipy's entr on random counters."""
    from scipy.special import entr
    E = 8
    # uniform load: exactly zero
    load = np.full(E, 5, np.int32)
    bias = orc.router_penalty(orc.ENTROPY, np.zeros((0, 1), np.int32), load, 0.9)
    assert (bias == 0).all()
    # nothing selected yet: zero (0 ln 0 = 0), and the first selections are absorbed first
    load = np.zeros(E, np.int32)
    bias = orc.router_penalty(orc.ENTROPY, np.zeros((0, 2), np.int32), load, 0.9)
    assert (bias == 0).all()
    bias = orc.router_penalty(orc.ENTROPY, np.array([[0, 1], [0, 2]], np.int32), load, 1.0)
    assert list(load) == [2, 1, 1, 0, 0, 0, 0, 0]
    p = load / load.sum()
    h = entr(p)
    np.testing.assert_allclose(bias, -(h - h.mean()), rtol=1e-6, atol=1e-9)
    # sign: shares 0.3 > 0.1: the busier expert gets the more negative term
    load = np.array([30, 10, 10, 10, 10, 10, 10, 10], np.int32)
    b1 = orc.router_penalty(orc.ENTROPY, np.zeros((0, 1), np.int32), load.copy(), 1.0)
    b3 = orc.router_penalty(orc.ENTROPY, np.zeros((0, 1), np.int32), load.copy(), 3.0)
    assert b1[0] < 0 < b1[1] and np.allclose(b1[1:], b1[1])
    np.testing.assert_allclose(b3, 3.0 * b1, rtol=1e-6)
    assert abs(float(b1.astype(np.float64).sum())) < 1e-6
    # random counters against the independent routine
    rng = np.random.default_rng(5)
    for _ in range(20):
        load = rng.integers(0, 1000, size=E).astype(np.int32)
        bias = orc.router_penalty(orc.ENTROPY, np.zeros((0, 1), np.int32), load, 0.37)
        h = entr(load / load.sum())
        np.testing.assert_allclose(bias, -0.37 * (h - h.mean()), rtol=1e-5, atol=1e-8)


def test_penalty_feeds_the_router_as_bias():
    """Closing the loop: a heavily loaded expert drops out of the top-k."""
    rng = np.random.default_rng(0)
    x = rng.standard_normal((1, 8)).astype(np.float32)
    W = rng.standard_normal((8, 4)).astype(np.float32)
    idx0, _, _ = orc.route(x, W, 1)
    load = np.zeros(4, np.int32)
    load[idx0[0, 0]] = 1000
    bias = orc.router_penalty(orc.LB, np.zeros((0, 1), np.int32), load, 1.0)
    idx1, _, _ = orc.route(x, W, 1, bias=bias)
    assert idx1[0, 0] != idx0[0, 0]


# ------------------------------------------------------------ compress on insert
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_compress_is_a_matmul_with_the_encoder(dtype):
    rng = np.random.default_rng(1)
    B, Hkv, D, r = 3, 2, 16, 4
    x = wl.encode(rng.standard_normal((B, Hkv, D)), dtype)
    W = wl.encode(rng.standard_normal((Hkv, r, D)) / 4, dtype)
    codes = orc.compress(x, W, dtype=dtype)
    ref = np.einsum("bhd,hcd->bhc", wl.decode(x, dtype).astype(np.float64), wl.decode(W, dtype).astype(np.float64))
    if dtype == "f32":
        np.testing.assert_allclose(codes, ref, rtol=1e-6)
    else:
        np.testing.assert_array_equal(codes, wl.f32_to_bf16_bits(ref.astype(np.float32)))


def test_compress_then_decode_with_orthonormal_rows_recovers_the_subspace():
    """Encoder = decoder^T with orthonormal rows: decode(encode(x)) is the projection of x, and a
    vector already in the row space comes back exactly (reconstruction error 0, Section 3.3)."""
    rng = np.random.default_rng(2)
    D, r = 16, 4
    Q, _ = np.linalg.qr(rng.standard_normal((D, r)))
    U = np.ascontiguousarray(Q.T[None].astype(np.float32))            # [1, r, D]
    inside = (rng.standard_normal((1, 1, r)) @ U[0]).astype(np.float32)   # in the row space
    codes = orc.compress(inside, U)
    np.testing.assert_allclose(codes[0, 0] @ U[0], inside[0, 0], rtol=1e-5, atol=1e-6)
    crop = np.zeros((1, r, D), np.float32)
    crop[0, np.arange(r), np.arange(r)] = 1                          # Table 2 "crop to r"
    x = rng.standard_normal((2, 1, D)).astype(np.float32)
    np.testing.assert_array_equal(orc.compress(x, crop), x[:, :, :r])


# ------------------------------------------------------------ scheduling policies (Table 3)
def _policy_state(B, E, S):
    return (np.zeros((B, E, S), np.int32), np.zeros((B, E, S), np.int32), np.zeros((B, E, S), np.int32))


def test_lru_eviction_drops_the_entries_accessed_longest_ago():
    """Table 3 row LRU (u = -recency) through the same eviction: the survivors are the `capacity`
    most recently accessed entries, found here by a plain sort of the access stamps."""
    rng = np.random.default_rng(5)
    B, E, S, cap, now = 2, 3, 40, 25, 1000
    birth, last, freq = _policy_state(B, E, S)
    last[:] = rng.integers(0, 900, size=(B, E, S))                       # repeated stamps: ties by slot
    last[0, 0, :] = rng.permutation(S) * 3                               # distinct stamps
    n = np.full((B, E), S, np.int32)
    u = orc.policy_utility(orc.POLICY_LRU, n, now, birth, last, freq)
    np.testing.assert_array_equal(u, -(now - last).astype(np.float32))
    ridx, rcnt = orc.evict(u.copy(), n.copy(), cap)
    for b in range(B):
        for e in range(E):
            order = sorted(range(S), key=lambda i: (last[b, e, i], -i))   # oldest first, higher slot first
            assert sorted(order[:S - cap]) == list(ridx[b, e, :rcnt[b, e]])


def test_lru_plus_interpolates_between_recency_and_frequency():
    rng = np.random.default_rng(6)
    B, E, S, now = 1, 2, 30, 500
    birth, last, freq = _policy_state(B, E, S)
    last[:] = rng.integers(0, now, size=(B, E, S))
    freq[:] = rng.integers(0, 50, size=(B, E, S))
    n = np.full((B, E), S, np.int32)
    lru = orc.policy_utility(orc.POLICY_LRU, n, now, birth, last, freq)
    # lambda = 0: the frequency term vanishes
    np.testing.assert_array_equal(orc.policy_utility(orc.POLICY_LRU_PLUS, n, now, birth, last, freq, lam=0.0), lru)
    # exact small-integer arithmetic: -r + 0.5 f is representable
    u = orc.policy_utility(orc.POLICY_LRU_PLUS, n, now, birth, last, freq, lam=0.5)
    np.testing.assert_array_equal(u, (-(now - last) + 0.5 * freq).astype(np.float32))
    # a large lambda orders by frequency first (least-frequently-used goes first)
    big = orc.policy_utility(orc.POLICY_LRU_PLUS, n, now, birth, last, freq, lam=1.0e4)
    ridx, rcnt = orc.evict(big.copy(), n.copy(), S - 5)
    for e in range(E):
        gone_f = freq[0, e, ridx[0, e, :5]]
        kept_f = np.delete(freq[0, e], ridx[0, e, :5])
        assert gone_f.max() <= kept_f.min()
    # the result is rounded once: a product that needs the fused form
    lam = np.float32(1.0 + 2.0 ** -12)
    freq[0, 0, 0], last[0, 0, 0] = 4097, now - 4097
    u = orc.policy_utility(orc.POLICY_LRU_PLUS, n, now, birth, last, freq, lam=float(lam))
    exact = float(lam) * 4097.0 - 4097.0                                  # exact in double
    assert u[0, 0, 0] == np.float32(exact) and u[0, 0, 0] != np.float32(np.float32(lam * np.float32(4097)) - np.float32(4097))


def test_sliding_window_policy_keeps_exactly_the_last_window_insertions():
    """Table 3 row SL: entries inserted one per step; after each insertion the shard is cut back to
    `window` entries with the indicator utility: what stays is the sliding window of the stream."""
    B, E, S, window = 1, 1, 12, 5
    birth, last, freq = _policy_state(B, E, S)
    n = np.zeros((B, E), np.int32)
    topk = np.zeros((1, 1), np.int32)
    reuse_idx = np.zeros((B, E, 1), np.int32)
    reuse_cnt = np.zeros((B, E), np.int32)
    for now in range(40):
        orc.policy_stamp(topk, n, now, birth, last, freq, reuse_idx, reuse_cnt)
        slot = reuse_idx[0, 0, 0] if reuse_cnt[0, 0] > 0 else n[0, 0]
        assert birth[0, 0, slot] == now and last[0, 0, slot] == now and freq[0, 0, slot] == 0
        n[0, 0] += 1                                     # the insert itself (a freed slot is refilled)
        reuse_cnt[:] = 0
        u = orc.policy_utility(orc.POLICY_SL, n, now, birth, last, freq, window=window)
        live = birth[0, 0, :n[0, 0]]
        np.testing.assert_array_equal(u[0, 0, :n[0, 0]], (now - live < window).astype(np.float32))
        if n[0, 0] > window:
            idx, cnt = orc.evict(u.copy(), n, window, max_evict=1)     # n becomes window: one hole
            assert cnt[0, 0] == 1
            reuse_idx[0, 0, 0], reuse_cnt[0, 0] = idx[0, 0, 0], 1
            hole = idx[0, 0, 0]
            kept = [birth[0, 0, i] for i in range(window + 1) if i != hole]
            assert sorted(kept) == list(range(now - window + 1, now + 1))


def test_protected_recent_entries_are_never_evicted():
    rng = np.random.default_rng(8)
    B, E, S, now, protect = 1, 2, 50, 200, 10
    birth, last, freq = _policy_state(B, E, S)
    birth[:] = rng.integers(150, now + 1, size=(B, E, S))
    last[:] = rng.integers(0, 100, size=(B, E, S))                       # young entries look stale to LRU
    n = np.full((B, E), S, np.int32)
    u = orc.policy_utility(orc.POLICY_LRU, n, now, birth, last, freq, protect=protect)
    young = now - birth < protect
    assert np.isposinf(u[young]).all() and np.isfinite(u[~young]).all()
    cap = int(young.sum(axis=2).max()) + 3
    ridx, rcnt = orc.evict(u.copy(), n.copy(), cap)
    for e in range(E):
        assert not young[0, e, ridx[0, e, :rcnt[0, e]]].any()
    # H2O passes the accumulated attention through (same shielding)
    h2o = rng.random((B, E, S)).astype(np.float32)
    u0 = orc.policy_utility(orc.POLICY_H2O, n, now, birth, last, freq, h2o=h2o)
    np.testing.assert_array_equal(u0, h2o)


def test_access_bookkeeping_counts_steps_above_the_threshold():
    rng = np.random.default_rng(9)
    B, E, S, steps, thr = 2, 2, 16, 25, 0.3
    birth, last, freq = _policy_state(B, E, S)
    last[:] = -1
    n = np.array([[16, 9], [0, 12]], np.int32)
    masses = rng.random((steps, B, E, S)).astype(np.float32)
    masses[3, 0, 0, 0] = thr                                             # equal is not above
    for t in range(steps):
        before = last.copy()
        orc.policy_access(masses[t], n, np.float32(thr), t, last, freq)
        hit = (masses[t] > np.float32(thr)) & (np.arange(S) < n[:, :, None])
        assert (last[hit] == t).all() and (last[~hit] == before[~hit]).all()
    live = np.arange(S) < n[:, :, None]
    above = masses > np.float32(thr)
    np.testing.assert_array_equal(freq, (above.sum(axis=0) * live).astype(np.int32))
    last_ref = np.where(above.any(axis=0), steps - 1 - np.argmax(above[::-1], axis=0), -1)
    np.testing.assert_array_equal(last[live], last_ref[live])
    assert (last[~live] == -1).all()


def test_policy_stamp_marks_the_slot_the_append_writes():
    """The bookkeeping call and the insert must agree on the slot: the entry whose utility the
    append resets is the entry stamped."""
    g = wl.Geometry(B=2, Hq=2, Hkv=2, D=8, E=3, S=6, k=2, dtype="f32")
    case = wl.make_host_case(g, seed=4, n_valid="ragged", utility0="exp")
    case.n_valid[:] = np.array([[6, 3, 0], [5, 4, 2]], np.int32)
    case.utility += 1.0
    topk = np.array([[0, 1], [1, 2]], np.int32)
    reuse_idx = np.zeros((g.B, g.E, 1), np.int32)
    reuse_cnt = np.zeros((g.B, g.E), np.int32)
    reuse_idx[0, 0, 0], reuse_cnt[0, 0] = 4, 1                         # shard (0,0) is full, slot 4 freed
    case.n_valid[0, 0] = 5
    birth, last, freq = _policy_state(g.B, g.E, g.S)
    birth[:], last[:], freq[:] = -5, -5, 9
    orc.policy_stamp(topk, case.n_valid, 77, birth, last, freq, reuse_idx, reuse_cnt)
    K_new, V_new = wl.draw_new_kv(g, seed=1)
    u = case.utility.copy()
    orc.append(K_new, V_new, topk, case.K_shards, case.V_shards, u, case.n_valid.copy(), dtype=g.dtype,
               reuse_idx=reuse_idx, reuse_cnt=reuse_cnt)
    stamped = birth == 77
    np.testing.assert_array_equal(stamped, (u == 0) & (case.utility != 0))
    assert (last[stamped] == 77).all() and (freq[stamped] == 0).all()
    assert (birth[~stamped] == -5).all() and (freq[~stamped] == 9).all()
    assert stamped.sum() == 4 and stamped[0, 0, 4] and stamped[0, 1, 3] and stamped[1, 1, 4] and stamped[1, 2, 2]
    full = np.full((g.B, g.E), g.S, np.int32)
    with pytest.raises(ValueError):                                     # no room: an error, as for the append
        orc.policy_stamp(topk, full, 78, birth, last, freq)


def test_rank_r_compressor_at_the_svd_optimum_leaves_the_tail_singular_values():
    """Table 2, rows LoRA / truncated SVD: with the encoder = decoder^T = the top-r right singular
    vectors, the squared reconstruction error of a set of rows is the sum of the squared singular
    values beyond r; the crop compressor's error is the energy of the dropped coordinates."""
    rng = np.random.default_rng(3)
    n, D, r = 12, 16, 5
    K = (rng.standard_normal((n, D)) * np.linspace(3.0, 0.2, D)).astype(np.float32)
    _, sig, Vt = np.linalg.svd(K.astype(np.float64), full_matrices=False)
    U = np.ascontiguousarray(Vt[:r][None].astype(np.float32))               # [1, r, D]
    codes = orc.compress(np.ascontiguousarray(K[:, None, :]), U)            # rows as a batch of 1-head tokens
    recon = codes[:, 0, :].astype(np.float64) @ U[0].astype(np.float64)
    err = ((K.astype(np.float64) - recon) ** 2).sum()
    np.testing.assert_allclose(err, (sig[r:] ** 2).sum(), rtol=1e-4)
    crop = np.zeros((1, r, D), np.float32)
    crop[0, np.arange(r), np.arange(r)] = 1
    kept = orc.compress(np.ascontiguousarray(K[:, None, :]), crop)[:, 0, :]
    err_crop = ((K[:, :r] - kept) ** 2).sum() + (K[:, r:].astype(np.float64) ** 2).sum()
    np.testing.assert_allclose(err_crop, (K[:, r:].astype(np.float64) ** 2).sum(), rtol=1e-12)
    assert err <= err_crop            # the SVD basis is the optimal rank-r choice


def test_policy_arrays_follow_a_compacting_eviction():
    """After evict(compact) + policy_compact, slot i of every array describes the same entry as the
    compacted utility at slot i: tag each entry with a unique id in all arrays and compare."""
    rng = np.random.default_rng(21)
    B, E, S, cap = 2, 3, 30, 17
    n = np.array([[30, 20, 17], [5, 30, 0]], np.int32)
    ids = np.arange(B * E * S, dtype=np.int32).reshape(B, E, S)
    u = ids.astype(np.float32) % 7 + rng.random((B, E, S)).astype(np.float32)   # distinct utilities
    tag_of = {float(u[b, e, i]): int(ids[b, e, i]) for b in range(B) for e in range(E) for i in range(S)}
    birth, last, freq = ids.copy(), ids.copy() + 1000, ids.copy() + 2000
    dummyK = [np.zeros((1, S, 4), np.float32) for _ in range(B * E)]
    dummyV = [np.zeros((1, S, 4), np.float32) for _ in range(B * E)]
    n_after = n.copy()
    eidx, ecnt = orc.evict(u, n_after, cap, compact=True, K_shards=dummyK, V_shards=dummyV, Hkv=1, width=4,
                           dtype="f32")
    orc.policy_compact(eidx, ecnt, n_after, birth, last, freq)
    for b in range(B):
        for e in range(E):
            for i in range(n_after[b, e]):
                tag = tag_of[float(u[b, e, i])]
                assert (birth[b, e, i], last[b, e, i], freq[b, e, i]) == (tag, tag + 1000, tag + 2000)
    assert (ecnt == np.maximum(n - cap, 0)).all()


def test_round_robin_router_is_exactly_balanced_and_selects_distinct_experts():
    """Table 1 row B: over any E consecutive (step, row) pairs every expert is taken k times; the k
    selections of one row are distinct; gates are uniform; routed attention accepts the result."""
    E, k, rows = 7, 3, 2
    counts = np.zeros(E, int)
    for step in range(100, 100 + E):
        idx, gates = orc.route_round_robin(rows, E, k, step)
        assert idx.shape == (rows, k) and (gates == np.float32(1.0 / k)).all()
        for r in range(rows):
            assert len(set(idx[r])) == k and idx[r].min() >= 0 and idx[r].max() < E
        counts += np.bincount(idx[0], minlength=E)
    assert (counts == k).all()
    a, _ = orc.route_round_robin(3, E, k, 5)
    b, _ = orc.route_round_robin(3, E, k, 6)
    np.testing.assert_array_equal(a[1:], b[:2])          # row r at step t = row r-1 at step t+1
    assert list(a[0]) == [(5 * k + j) % E for j in range(k)]



# ------------------------------------------------------------ decoder bias of the values
def test_value_decoder_bias_adds_the_same_vector_to_every_output():
    """Table 2 row LoRA++: reconstruction W_d W_u x + b.  On the value side every decoded entry
    gains b[h'], and since the attention weights of a row sum to one, so does every output row
    with a non-empty selection (an empty one stays zero).  Probabilities and utilities do not
    move.  Against an independent numpy attention over explicitly decoded entries as well."""
    g = wl.Geometry(B=2, Hq=4, Hkv=2, D=16, E=3, S=10, k=2, dtype="f32", rank=4)
    case = wl.make_host_case(g, seed=8, n_valid="ragged")
    case.n_valid[1, :] = 0                                  # sequence 1: every shard empty
    rng = np.random.default_rng(9)
    b_V = rng.standard_normal((g.Hkv, g.D)).astype(np.float32)
    idx = np.array([[0, 2], [1, 2]], np.int32)
    gates = np.array([[0.7, 0.3], [0.5, 0.5]], np.float32)
    for combine in (orc.COMBINE_LSE, orc.COMBINE_LOCAL):
        u0, u1 = case.utility.copy(), case.utility.copy()
        kw = dict(Hkv=g.Hkv, E=g.E, S=g.S, dtype=g.dtype, rank=g.rank, U_K=case.U_K, U_V=case.U_V,
                  combine=combine, want_prob=True)
        plain = orc.attend(case.q, case.K_shards, case.V_shards, case.n_valid, idx, gates, utility=u0, **kw)
        biased = orc.attend(case.q, case.K_shards, case.V_shards, case.n_valid, idx, gates, utility=u1,
                            V_bias=b_V, **kw)
        G = g.Hq // g.Hkv
        for h in range(g.Hq):
            np.testing.assert_allclose(biased["y"][0, h] - plain["y"][0, h], b_V[h // G], rtol=1e-5, atol=1e-6)
        assert (biased["y"][1] == 0).all() and (plain["y"][1] == 0).all()
        np.testing.assert_array_equal(biased["prob"], plain["prob"])
        np.testing.assert_array_equal(u0, u1)
    # independent check of the biased output in LSE mode with unit gates: dense attention over the
    # concatenation of the two selected shards, entries decoded explicitly
    ones = np.ones_like(gates)
    out = orc.attend(case.q, case.K_shards, case.V_shards, case.n_valid, idx, ones, Hkv=g.Hkv, E=g.E, S=g.S,
                     dtype=g.dtype, rank=g.rank, U_K=case.U_K, U_V=case.U_V, V_bias=b_V)
    G = g.Hq // g.Hkv
    for h in range(g.Hq):
        hk = h // G
        Kd = np.concatenate([case.K_shards[e][hk, :case.n_valid[0, e]].astype(np.float64) @ case.U_K[hk]
                             for e in idx[0]])
        Vd = np.concatenate([case.V_shards[e][hk, :case.n_valid[0, e]].astype(np.float64) @ case.U_V[hk]
                             + b_V[hk] for e in idx[0]])
        sc = Kd @ case.q[0, h].astype(np.float64) / np.sqrt(g.D)
        w = np.exp(sc - sc.max())
        np.testing.assert_allclose(out["y"][0, h], (w / w.sum()) @ Vd, rtol=1e-5, atol=1e-6)
