"""The C-ABI library loads without a GPU, exports every function the header declares, and
rejects bad arguments on the host before anything is launched."""
import ctypes as C
import os
import re

import pytest

import paper_2508_06526_amd as pk
from paper_2508_06526_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "pikv.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pikv_[a-z_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(pk.library_path()):
        from paper_2508_06526_amd import build
        build.build()
    return pk.load_library()


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_strerror(lib):
    assert pk.pikv_version() >= 100
    assert pk.pikv_strerror(0) == "ok"
    for code in (-1, -2, -3, -4, 77):
        assert pk.pikv_strerror(code)


def test_desc_struct_matches_header_layout():
    assert C.sizeof(pk.PikvDesc) == 64
    assert pk.PikvDesc.stride_h.offset == 32 and pk.PikvDesc.route_rows_per_seq.offset == 48
    assert pk.PikvDesc.flags.offset == 52 and pk.PikvDesc.tq.offset == 56


def test_workspace_size_is_zero_for_bad_geometry_and_positive_otherwise(lib):
    good = pk.make_desc(1, 32, 8, 128, 16, 8192)
    assert pk.pikv_attn_workspace_bytes(good, 4) > 0
    assert pk.pikv_attn_workspace_bytes(good, 0) == 0
    assert pk.pikv_attn_workspace_bytes(good, 17) == 0
    assert pk.pikv_attn_workspace_bytes(pk.make_desc(1, 32, 5, 128, 16, 8192), 4) == 0   # Hq % Hkv
    assert pk.pikv_attn_workspace_bytes(pk.make_desc(1, 32, 8, 96, 16, 8192), 4) == 0    # D
    assert pk.pikv_attn_workspace_bytes(pk.make_desc(1, 32, 8, 128, 65, 8192), 4) == 0   # E > 64
    assert pk.pikv_attn_workspace_bytes(pk.make_desc(1, 32, 8, 128, 16, 8192, rank=24), 4) == 0


def test_host_side_argument_errors(lib):
    """NULL pointers / out-of-range sizes return PIKV_ERR_INVALID with no GPU present."""
    vp = C.c_void_p
    fake = vp(0x1000)        # never dereferenced: every call below fails validation first
    INVALID, UNSUPPORTED, WORKSPACE = -1, -2, -3
    r = lib.pikv_route
    assert r(None, fake, None, 1, 8, 4, 2, 0, fake, fake, None, None) == INVALID
    assert r(fake, fake, None, 1, 8, 4, 5, 0, fake, fake, None, None) == INVALID      # k > E
    assert r(fake, fake, None, 1, 8, 65, 2, 0, fake, fake, None, None) == INVALID     # E > 64
    assert r(fake, fake, None, 1, 0, 4, 2, 0, fake, fake, None, None) == INVALID      # d_r
    assert r(fake, fake, None, 1, 8, 4, 2, 9, fake, fake, None, None) == INVALID      # dtype
    assert r(fake, fake, None, 0, 8, 4, 2, 0, fake, fake, None, None) == 0            # no rows

    d = pk.make_desc(1, 4, 4, 64, 4, 256)
    a = lib.pikv_sharded_attn

    def attn(desc, q=fake, k=2, combine=0, ws=fake, ws_bytes=1 << 30, y=fake, uk=None):
        return a(C.byref(desc), q, fake, fake, uk, uk, fake, fake, None, k, combine, 0.0, y, None,
                 None, None, None, ws, ws_bytes, None)
    assert attn(d, q=None) == INVALID
    assert attn(d, y=None) == INVALID
    assert attn(d, k=0) == INVALID
    assert attn(d, combine=3) == INVALID
    assert attn(d, ws_bytes=16) == WORKSPACE
    assert attn(d, ws=None) == WORKSPACE
    assert attn(pk.make_desc(1, 4, 4, 64, 4, 256, rank=32)) == INVALID                 # U_K missing
    assert attn(pk.make_desc(1, 4, 4, 48, 4, 256)) == UNSUPPORTED
    assert attn(pk.make_desc(1, 4, 4, 64, 4, 256, stride_s=60)) == INVALID
    assert attn(pk.make_desc(1, 4, 4, 64, 4, 256, route_rows_per_seq=2)) == INVALID
    assert attn(pk.make_desc(0, 4, 4, 64, 4, 256)) == 0                                # B == 0

    u = lib.pikv_update_utility
    assert u(C.byref(d), None, fake, fake, fake, 2, 1.0, fake, None) == INVALID
    assert u(C.byref(d), fake, fake, fake, fake, 2, -0.5, fake, None) == INVALID
    assert u(C.byref(d), fake, fake, fake, fake, 9, 1.0, fake, None) == INVALID
    assert u(C.byref(d), fake, fake, fake, fake, 2, float("nan"), fake, None) == INVALID

    e = lib.pikv_evict
    assert e(C.byref(d), None, fake, 10, None, 0, fake, fake, 4, 0, None, None, None) == INVALID
    assert e(C.byref(d), fake, fake, -1, None, 0, fake, fake, 4, 0, None, None, None) == INVALID
    assert e(C.byref(d), fake, fake, 10, None, 0, fake, fake, 0, 0, None, None, None) == INVALID
    assert e(C.byref(d), fake, fake, 10, fake, 0, fake, fake, 4, 0, None, None, None) == INVALID
    assert e(C.byref(d), fake, fake, 10, None, 0, fake, fake, 4, 1, None, None, None) == INVALID

    ap = lib.pikv_append
    assert ap(C.byref(d), None, fake, fake, 2, None, None, 0, fake, fake, fake, fake, None) == INVALID
    assert ap(C.byref(d), fake, fake, fake, 5, None, None, 0, fake, fake, fake, fake, None) == INVALID
    assert ap(C.byref(d), fake, fake, fake, 2, fake, None, 1, fake, fake, fake, fake, None) == INVALID


def test_host_side_argument_errors_of_the_widened_entry_points(lib):
    vp = C.c_void_p
    fake = vp(0x1000)        # never dereferenced
    INVALID, UNSUPPORTED, WORKSPACE = -1, -2, -3
    d = pk.make_desc(2, 4, 4, 64, 8, 256, dtype=1)

    def step(desc=d, q=fake, K_new=fake, V_new=fake, eidx=fake, k=2, decay=1.0, combine=0, ws=fake,
             ws_bytes=1 << 30, scores=fake, scale=0.0, U=None):
        return lib.pikv_decode_step(C.byref(desc), q, fake, None, K_new, V_new, fake, fake, U, U, fake,
                                    fake, k, combine, scale, decay, fake, fake, eidx, fake, fake, None, None,
                                    scores, fake, ws, ws_bytes, None)
    assert step(q=None) == INVALID
    assert step(V_new=None) == INVALID                     # K_new without V_new
    assert step(eidx=None) == INVALID                      # insert without the eviction outputs
    assert step(k=0) == INVALID and step(k=9) == INVALID
    assert step(decay=-1.0) == INVALID and step(combine=2) == INVALID
    assert step(scores=None) == INVALID
    assert step(ws_bytes=8) == WORKSPACE
    # the checks of the attention pass are made before the step's first launch as well
    assert step(ws=vp(0x1010)) == INVALID                  # workspace not 256-byte aligned
    assert step(scale=float("nan")) == INVALID
    assert step(desc=pk.make_desc(2, 4, 4, 64, 8, 256, rank=32, dtype=1)) == INVALID   # codes without decoders
    assert step(desc=pk.make_desc(2, 4, 4, 64, 8, 256, dtype=1, route_rows_per_seq=4)) == UNSUPPORTED
    assert step(desc=pk.make_desc(0, 4, 4, 64, 4, 256, dtype=1)) == 0   # W_r rows of 8 bytes: accepted (nothing to launch)
    assert step(desc=pk.make_desc(0, 4, 4, 64, 8, 256, dtype=1)) == 0

    rr = lib.pikv_route_round_robin
    rr.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int64, vp, vp, vp]
    assert rr(2, 8, 9, 0, fake, fake, None) == INVALID
    assert rr(2, 65, 2, 0, fake, fake, None) == INVALID
    assert rr(2, 8, 2, -1, fake, fake, None) == INVALID
    assert rr(2, 8, 2, 0, None, fake, None) == INVALID
    assert rr(0, 8, 2, 0, fake, fake, None) == 0

    rp = lib.pikv_router_penalty
    assert rp(7, fake, 1, 2, 8, fake, None, 0.1, fake, None) == INVALID
    assert rp(3, fake, 1, 2, 8, fake, None, 0.1, fake, None) == INVALID           # modes are 0, 1, 2
    assert rp(0, fake, 1, 2, 8, None, None, 0.1, fake, None) == INVALID
    assert rp(0, fake, 1, 2, 65, fake, None, 0.1, fake, None) == INVALID
    assert rp(1, fake, 1, 2, 8, fake, None, 0.1, fake, None) == INVALID           # cache-aware needs miss
    assert rp(0, fake, 1, 2, 8, fake, None, float("nan"), fake, None) == INVALID

    cp = lib.pikv_compress
    dr = pk.make_desc(2, 4, 4, 64, 8, 256, rank=32, dtype=1)
    assert cp(C.byref(d), fake, fake, fake, None, None, None, None) == INVALID    # rank == 0
    assert cp(C.byref(dr), None, fake, fake, None, None, None, None) == INVALID
    assert cp(C.byref(dr), fake, fake, fake, fake, None, None, None) == INVALID   # partly given V

    st = lib.pikv_policy_stamp
    assert st(C.byref(d), None, 2, None, None, 0, fake, 5, fake, fake, fake, None) == INVALID
    assert st(C.byref(d), fake, 9, None, None, 0, fake, 5, fake, fake, fake, None) == INVALID
    assert st(C.byref(d), fake, 2, fake, None, 1, fake, 5, fake, fake, fake, None) == INVALID
    assert st(C.byref(d), fake, 2, fake, fake, 0, fake, 5, fake, fake, fake, None) == INVALID
    assert st(C.byref(pk.make_desc(2, 4, 4, 64, 8, 256, dtype=1, route_rows_per_seq=4)), fake, 2, None, None, 0,
              fake, 5, fake, fake, fake, None) == UNSUPPORTED

    tr = lib.pikv_update_utility_tracked
    assert tr(C.byref(d), fake, fake, fake, fake, 2, 1.0, None, 0.1, 5, None, fake, None) == INVALID
    assert tr(C.byref(d), fake, fake, fake, fake, 2, 1.0, None, -0.1, 5, fake, fake, None) == INVALID
    assert tr(C.byref(d), fake, fake, fake, fake, 2, -1.0, fake, 0.1, 5, fake, fake, None) == INVALID
    assert tr(C.byref(pk.make_desc(0, 4, 4, 64, 8, 256, dtype=1)), fake, fake, fake, fake, 2, 1.0, None, 0.1, 5,
              fake, fake, None) == 0

    lib.pikv_decode_step_policy.argtypes = list(lib.pikv_decode_step.argtypes) + [vp, vp]
    lib.pikv_decode_step_policy.restype = C.c_int

    def pstep(args):
        return lib.pikv_decode_step_policy(C.byref(d), fake, fake, None, fake, fake, fake, fake, None, None, fake,
                                           fake, 2, 0, 0.0, 1.0, fake, fake, fake, fake, fake, None, None, fake,
                                           fake, fake, 1 << 30, None, C.cast(C.pointer(args), vp), None)
    fakeptr = 0x1000
    bad = pk.PikvPolicyArgs(policy=9, now=1)
    assert pstep(bad) == INVALID
    assert pstep(pk.PikvPolicyArgs(policy=pk.POLICY_LRU, now=1)) == INVALID                     # needs last_access
    assert pstep(pk.PikvPolicyArgs(policy=pk.POLICY_SL, now=1, window=4)) == INVALID             # needs birth
    assert pstep(pk.PikvPolicyArgs(policy=pk.POLICY_LRU, now=1, last_access=fakeptr, freq=fakeptr,
                                   threshold=-1.0)) == INVALID                                   # tracking threshold
    assert pstep(pk.PikvPolicyArgs(policy=pk.POLICY_LRU_PLUS, now=1, lam=float("nan"), last_access=fakeptr,
                                   freq=fakeptr)) == INVALID
    def fstep(fb):
        return lib.pikv_decode_step_policy(C.byref(d), fake, fake, None, fake, fake, fake, fake, None, None, fake,
                                           fake, 2, 0, 0.0, 1.0, fake, fake, fake, fake, fake, None, None, fake,
                                           fake, fake, 1 << 30, None, None, C.cast(C.pointer(fb), vp))
    assert fstep(pk.PikvRouterFeedback(mode=5, coef=0.1, load=fakeptr, bias=fakeptr)) == INVALID
    assert fstep(pk.PikvRouterFeedback(mode=0, coef=0.1, load=None, bias=fakeptr)) == INVALID
    assert fstep(pk.PikvRouterFeedback(mode=1, coef=0.1, load=fakeptr, bias=fakeptr)) == INVALID   # needs miss
    assert fstep(pk.PikvRouterFeedback(mode=2, coef=float("nan"), load=fakeptr, bias=fakeptr)) == INVALID
    # descriptor flags: only the value-bias bit, and only with codes
    assert step(desc=pk.make_desc(2, 4, 4, 64, 8, 256, dtype=1, flags=1)) == INVALID
    assert step(desc=pk.make_desc(2, 4, 4, 64, 8, 256, dtype=1, flags=2)) == INVALID
    pc = lib.pikv_policy_compact
    assert pc(C.byref(d), None, fake, 4, fake, fake, fake, fake, None) == INVALID
    assert pc(C.byref(d), fake, fake, 0, fake, fake, fake, fake, None) == INVALID
    assert pc(C.byref(pk.make_desc(0, 4, 4, 64, 8, 256, dtype=1)), fake, fake, 4, fake, fake, fake, fake, None) == 0

    pu = lib.pikv_policy_utility
    assert pu(C.byref(d), 4, fake, 5, 0.0, 0, 0, fake, fake, fake, fake, fake, None) == INVALID
    assert pu(C.byref(d), 0, fake, 5, 0.0, 0, 0, fake, fake, fake, None, fake, None) == INVALID   # H2O needs h2o
    assert pu(C.byref(d), 1, fake, 5, 0.0, 3, 0, None, fake, fake, None, fake, None) == INVALID   # SL needs birth
    assert pu(C.byref(d), 2, fake, 5, 0.0, 0, 0, fake, None, fake, None, fake, None) == INVALID   # LRU needs last
    assert pu(C.byref(d), 3, fake, 5, float("nan"), 0, 0, fake, fake, fake, None, fake, None) == INVALID
    assert pu(C.byref(d), 2, fake, 5, 0.0, -1, 0, fake, fake, fake, None, fake, None) == INVALID
    assert pu(C.byref(d), 2, fake, 5, 0.0, 0, 2, None, fake, fake, None, fake, None) == INVALID   # protect needs birth
    assert pu(C.byref(d), 2, fake, 5, 0.0, 0, 0, None, fake, None, None, None, None) == INVALID   # out


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(OSError):
        binding.load_library()
