"""Shared plumbing of the GPU parity tests: upload a host case, run the HIP path through the
C-ABI binding, bring results back as numpy.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch

import paper_2508_06526_amd as pk
import workloads as wl
from oracle import pikv_oracle as orc

DEV = "cuda:0"


def dev_storage(a: np.ndarray, dtype: str) -> torch.Tensor:
    """numpy storage array (f32, or bf16 bits as uint16) -> device tensor of that dtype."""
    if dtype == "f32":
        return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    t = torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(DEV)
    return t.view(torch.bfloat16)


def host_storage(t: torch.Tensor, dtype: str) -> np.ndarray:
    return wl.to_host(t, dtype)


class DeviceCase:
    """Device copy of a workloads.HostCase plus the output/scratch buffers of one step."""

    def __init__(self, case: wl.HostCase, k=None, stride_pad=(0, 0)):
        g = case.geo
        self.geo = g
        self.k = g.k if k is None else k
        dt = g.dtype
        self.q = dev_storage(case.q, dt)
        self.W_r = dev_storage(case.W_r, dt)
        self.bias = None if case.bias is None else torch.from_numpy(case.bias).to(DEV)
        pad_s, pad_rows = stride_pad
        w = g.width
        self.stride_s = w + pad_s
        self.stride_h = (g.S + pad_rows) * self.stride_s
        tdt = torch.float32 if dt == "f32" else torch.bfloat16
        shape = (g.B * g.E, g.Hkv, g.S + pad_rows, w + pad_s)
        self.K = torch.zeros(shape, device=DEV, dtype=tdt)
        self.V = torch.zeros(shape, device=DEV, dtype=tdt)
        for i in range(g.B * g.E):
            self.K[i, :, :g.S, :w] = dev_storage(case.K_shards[i], dt)
            self.V[i, :, :g.S, :w] = dev_storage(case.V_shards[i], dt)
        self.K_tab = pk.shard_table([self.K[i] for i in range(g.B * g.E)])
        self.V_tab = pk.shard_table([self.V[i] for i in range(g.B * g.E)])
        self.U_K = None if case.U_K is None else dev_storage(case.U_K, dt)
        self.U_V = None if case.U_V is None else dev_storage(case.U_V, dt)
        self.n_valid = torch.from_numpy(case.n_valid).to(DEV)
        self.utility = torch.from_numpy(case.utility).to(DEV)
        self.desc = pk.make_desc(g.B, g.Hq, g.Hkv, g.D, g.E, g.S, rank=g.rank,
                                 dtype=pk.binding.F32 if dt == "f32" else pk.binding.BF16,
                                 stride_h=self.stride_h, stride_s=self.stride_s,
                                 route_rows_per_seq=g.Hq if g.per_head_routing else 1)
        R, k = g.route_rows, self.k
        self.topk = torch.zeros((R, k), device=DEV, dtype=torch.int32)
        self.gates = torch.zeros((R, k), device=DEV, dtype=torch.float32)
        self.probs = torch.zeros((R, g.E), device=DEV, dtype=torch.float32)
        self.y = torch.full((g.B, g.Hq, g.D), float("nan"), device=DEV)
        self.row_max = torch.zeros((g.B, g.Hq), device=DEV)
        self.row_norm = torch.zeros((g.B, g.Hq), device=DEV)
        self.scores = torch.full((g.B, g.Hq, k, g.S), float("nan"), device=DEV)
        self.slot_coef = torch.zeros((g.B, g.Hq, k, 2), device=DEV)
        nbytes = pk.pikv_attn_workspace_bytes(self.desc, k)
        assert nbytes > 0
        self.workspace = torch.empty(nbytes, device=DEV, dtype=torch.uint8)

    # ---- the calls, each straight through the binding
    def route(self, x=None):
        g = self.geo
        x = wl.routing_rows(g, self.q) if x is None else x
        pk.pikv_route(x, self.W_r, self.bias, g.route_rows, g.d_r, g.E, self.k, self.topk,
                      self.gates, self.probs)

    def attend(self, topk=None, gates="own", combine=pk.COMBINE_LSE, scale=0.0, want_scores=True):
        topk = self.topk if topk is None else topk
        if isinstance(gates, str):
            gates = self.gates
        pk.pikv_sharded_attn(self.desc, self.q, self.K_tab, self.V_tab, self.U_K, self.U_V,
                             self.n_valid, topk, gates, self.k, combine, scale, self.y,
                             self.row_max, self.row_norm, self.scores if want_scores else None,
                             self.slot_coef if want_scores else None, self.workspace)

    def update_utility(self, decay, topk=None):
        topk = self.topk if topk is None else topk
        pk.pikv_update_utility(self.desc, self.scores, self.slot_coef, self.n_valid, topk, self.k,
                               decay, self.utility)

    def shard_host(self, which, i):
        g = self.geo
        t = (self.K if which == "K" else self.V)[i, :, :g.S, :g.width].contiguous()
        return host_storage(t, g.dtype)


def t2n(t):
    torch.cuda.synchronize()
    return t.detach().cpu().numpy().copy()


def y_tolerance_ok(y_gpu, y_ref, dtype):
    """bf16 storage: |d| <= 2e-3 + 1e-2 |ref| and relative L2 <= 1e-3; fp32 storage: 2e-5 / 1e-4."""
    if dtype == "f32":
        atol, rtol, l2 = 2e-5, 1e-4, 1e-5
    else:
        atol, rtol, l2 = 2e-3, 1e-2, 1e-3
    err = np.abs(y_gpu - y_ref)
    ok_elem = bool((err <= atol + rtol * np.abs(y_ref)).all())
    den = np.linalg.norm(y_ref)
    ok_l2 = True if den == 0 else bool(np.linalg.norm(y_gpu - y_ref) / den <= l2)
    return ok_elem and ok_l2, float(err.max()), float(np.linalg.norm(y_gpu - y_ref) / max(den, 1e-30))


def assert_utility_close(u_gpu, u_ref):
    np.testing.assert_allclose(u_gpu, u_ref, rtol=1e-4, atol=1e-9)


def ensure_route_margin(case: wl.HostCase, k: int, margin: float = 1e-3, max_redraw: int = 50):
    """Redraw query rows whose k-th and (k+1)-th logits (fp64, from the oracle) are closer
    than `margin`, so that any fp32 summation order selects the same experts."""
    g = case.geo
    if g.E == 1:
        return
    for attempt in range(max_redraw):
        x = wl.routing_rows(g, case.q)
        _, _, _, logits = orc.route(np.ascontiguousarray(x), case.W_r, k, bias=case.bias,
                                    dtype=g.dtype, want_logits=True)
        srt = -np.sort(-logits, axis=1)
        # adjacent pairs among the first k+1: the selection AND its output order are decided there
        gaps = np.abs(np.diff(srt[:, :k + 1], axis=1)).min(axis=1)
        bad = np.nonzero(gaps < margin)[0]
        if bad.size == 0:
            return
        # a routed row is a whole sequence (or one head of it): all its queries are redrawn
        fresh = wl.draw_queries(g, 10_000 + attempt).reshape(g.route_rows, -1)
        q = case.q.reshape(g.route_rows, -1).copy()
        q[bad] = fresh[bad]
        case.q = np.ascontiguousarray(q.reshape(g.B, g.Hq, g.D))
    raise AssertionError("could not reach the routing margin")
