"""The attention entry point that allocates nothing (its split partials live in a fixed array
inside the library's device image) against pikv_sharded_attn with a caller workspace: same
kernels, so every output must carry the same bits - on two calls in a row, the second on a
smaller input, so that what the first call left in the shared array cannot leak into it."""
import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():  # pragma: no cover
    pytest.skip("no GPU", allow_module_level=True)

import paper_2508_06526_amd as pk  # noqa: E402
from gpu_harness import DEV, DeviceCase, ensure_route_margin, t2n  # noqa: E402
from oracle import pikv_oracle as orc  # noqa: E402
from gpu_harness import y_tolerance_ok  # noqa: E402


def run_both(spec, seed, combine):
    g = wl.Geometry(**spec)
    case = wl.make_host_case(g, seed=seed, zipf_s=1.1)
    case.n_valid[:, 1] = max(1, g.S // 3)          # a ragged shard: some splits stay empty
    ensure_route_margin(case, g.k)
    a, b = DeviceCase(case), DeviceCase(case)
    a.route()
    b.route()
    a.attend(combine=combine)                       # caller workspace
    pk.pikv_sharded_attn_noalloc(b.desc, b.q, b.K_tab, b.V_tab, b.U_K, b.U_V, b.n_valid, b.topk, b.gates,
                                 b.k, combine, 0.0, b.y, b.row_max, b.row_norm, b.scores, b.slot_coef)
    torch.cuda.synchronize()
    for name in ("y", "row_max", "row_norm", "slot_coef"):
        np.testing.assert_array_equal(t2n(getattr(a, name)).view(np.uint32), t2n(getattr(b, name)).view(np.uint32),
                                      err_msg=name)
    # visited score rows only (the rest of the scratch is never written by either call)
    sa, sb = t2n(a.scores), t2n(b.scores)
    live = ~np.isnan(sa)
    assert (live == ~np.isnan(sb)).all()
    np.testing.assert_array_equal(sa[live].view(np.uint32), sb[live].view(np.uint32))
    # and against the oracle, to the attention tolerance
    idx, gates = t2n(b.topk), t2n(b.gates)
    out = orc.attend(case.q, case.K_shards, case.V_shards, case.n_valid, idx, gates, Hkv=g.Hkv, E=g.E, S=g.S,
                     dtype=g.dtype, rank=g.rank, U_K=case.U_K, U_V=case.U_V, combine=combine)
    ok, emax, l2 = y_tolerance_ok(t2n(b.y), out["y"], g.dtype)
    assert ok, (emax, l2)


def test_no_alloc_attention_equals_the_workspace_call_on_two_calls_in_a_row():
    big = dict(B=2, Hq=8, Hkv=2, D=128, E=8, S=1500, k=3, dtype="bf16")        # matrix-core kernel, many splits
    small = dict(B=1, Hq=4, Hkv=4, D=64, E=4, S=200, k=2, dtype="f32")         # plain kernel, smaller partials
    run_both(big, 11, pk.COMBINE_LSE)
    run_both(small, 12, pk.COMBINE_LOCAL)
    run_both(dict(B=2, Hq=4, Hkv=4, D=128, E=8, S=300, k=2, dtype="bf16", rank=32), 13, pk.COMBINE_LSE)


def test_no_alloc_attention_rejects_a_geometry_beyond_its_fixed_scratch():
    g = wl.Geometry(B=64, Hq=32, Hkv=32, D=128, E=8, S=4096, k=8, dtype="bf16")
    desc = pk.make_desc(g.B, g.Hq, g.Hkv, g.D, g.E, g.S, dtype=1)
    assert pk.pikv_attn_workspace_bytes(desc, g.k) > pk.NOALLOC_SCRATCH_BYTES
    fake = torch.zeros(16, device=DEV)
    with pytest.raises(pk.PikvError) as err:
        pk.pikv_sharded_attn_noalloc(desc, fake, fake, fake, None, None, fake, fake, None, g.k, pk.COMBINE_LSE,
                                     0.0, fake, None, None, None, None)
    assert err.value.status == -3
