"""Glue for the GPU parity tests: move a numpy workload to the device, run the
HIP library through its binding, and bring the results back as numpy."""
import numpy as np
import torch

from paper_2605_08527_amd import api
from harness import workloads as wl

TOL_MAX, TOL_MEAN = 1e-2, 1e-3   # floored relative error vs the fp64 oracle (bf16 in, fp32 accumulate)


def to_dev(a):
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def to_host(t):
    if t.dtype == torch.bfloat16:
        return wl.bf16_bits_to_f32(t.view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)
    return t.cpu().numpy().astype(np.float64)


class HipLayer:
    """One workload resident on the GPU with its context, map and descriptor.  With table=True the
    adapters (and their gradient buffers) are registered in an adapter table object and the
    descriptor refers to it; otherwise the descriptor carries the host pointer lists."""

    def __init__(self, w, out_dtype=torch.float32, want_bwd=False, ctx=None, table=False, packed=False, kept_wt=False):
        self.w = w
        self.ctx = ctx or api.marlaas_create(0)
        self.x, self.W = to_dev(w["x"]), to_dev(w["W"])
        self.A = [to_dev(a) for a in w["A"]]
        self.B = [to_dev(b) for b in w["B"]]
        self.ids = torch.from_numpy(np.ascontiguousarray(w["ids"], dtype=np.int32)).cuda()
        self.dY = to_dev(w["dY"]) if w.get("dY") is not None else None
        self.n = len(self.A)
        self.map = api.marlaas_segmap_build(self.ctx, self.ids, self.n)
        self.table = None
        self.gA = self.gB = None
        self.Wp_fwd = self.Wp_bwd = None
        # a transposed copy of the frozen weight kept across calls (large batches read it where the
        # contraction runs along W's strided dimension)
        self.W_t = api.marlaas_transpose_weight(self.ctx, self.W, w["layout"]) if (kept_wt and w["dtype"] == "bf16") else None
        if packed and w["dtype"] == "bf16":          # packed copies of the frozen weight (small batches read them)
            self.Wp_fwd = api.marlaas_pack_weight(self.ctx, self.W, w["layout"], 0)
            if want_bwd:
                self.Wp_bwd = api.marlaas_pack_weight(self.ctx, self.W, w["layout"], 1)
        if table and self.n > 0:
            self.table = api.marlaas_adapter_table_create(self.ctx, self.n, 1, int(max(w["ranks"])))
            if want_bwd:
                self.gA = [torch.full(tuple(a.shape), float("nan"), dtype=torch.float32, device="cuda") for a in self.A]
                self.gB = [torch.full(tuple(b.shape), float("nan"), dtype=torch.float32, device="cuda") for b in self.B]
            for t in range(self.n):
                api.marlaas_adapter_table_update(self.ctx, self.table, 0, t, self.A[t], self.B[t], int(w["ranks"][t]),
                                                 float(w["scales"][t]), self.gA[t] if want_bwd else None,
                                                 self.gB[t] if want_bwd else None)
            self.desc = api.LoraDesc(self.x, self.W, None, None, None, None, self.map, layout=w["layout"],
                                     out_dtype=out_dtype, table=self.table, W_packed_fwd=self.Wp_fwd, W_packed_bwd=self.Wp_bwd, W_t=self.W_t)
        else:
            self.desc = api.LoraDesc(self.x, self.W, self.A, self.B, w["ranks"], w["scales"], self.map,
                                     layout=w["layout"], out_dtype=out_dtype, W_packed_fwd=self.Wp_fwd, W_packed_bwd=self.Wp_bwd, W_t=self.W_t)
        self.out_dtype = out_dtype
        nbytes = api.marlaas_workspace_bytes(self.desc, want_bwd)
        self.ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
        api.marlaas_set_workspace(self.ctx, self.ws)
        self.T, self.K, self.N = self.desc.shape[:3]

    def fwd(self, save_u=False):
        y = torch.full((self.T, self.N), float("nan"), dtype=self.out_dtype, device="cuda")
        u = None
        if save_u:
            u = torch.zeros((max(self.T, 1), api.marlaas_u_stride(self.desc)), dtype=torch.float32, device="cuda")
        api.marlaas_lora_fwd(self.ctx, self.desc, y, u_save=u)
        torch.cuda.synchronize()
        return y, u

    def bwd(self, u_saved=None, accumulate=False, init=None, want_dX=True, want_grads=True):
        dX = torch.full((self.T, self.K), float("nan"), dtype=self.out_dtype, device="cuda") if want_dX else None
        dA = dB = None
        fill = float("nan") if init is None else init
        if want_grads and self.table is not None:
            dA, dB = self.gA, self.gB
            for g in dA + dB:
                g.fill_(fill)
            api.marlaas_lora_bwd(self.ctx, self.desc, self.dY, dX=dX, dA=api.MARLAAS_GRADS_IN_TABLE,
                                 dB=api.MARLAAS_GRADS_IN_TABLE, u_saved=u_saved, accumulate=accumulate)
        else:
            if want_grads:
                dA = [torch.full(tuple(a.shape), fill, dtype=torch.float32, device="cuda") for a in self.A]
                dB = [torch.full(tuple(b.shape), fill, dtype=torch.float32, device="cuda") for b in self.B]
            api.marlaas_lora_bwd(self.ctx, self.desc, self.dY, dX=dX, dA=dA, dB=dB, u_saved=u_saved,
                                 accumulate=accumulate)
        torch.cuda.synchronize()
        return dX, dA, dB


def oracle_grads_in_layout(dA, dB, layout):
    """Oracle gradients are in math orientation; transpose for the torch layout."""
    if layout == 1:
        return [a.T for a in dA], [b.T for b in dB]
    return dA, dB


def assert_close(got, ref, what, tol_max=TOL_MAX, tol_mean=TOL_MEAN):
    mx, mean, nrm = wl.rel_err_stats(got, ref)
    assert np.all(np.isfinite(got)), "%s has non-finite values" % what
    assert mx <= tol_max and mean <= tol_mean, "%s: max rel %.3e mean rel %.3e norm %.3e" % (what, mx, mean, nrm)
    return mx, mean


def bf16_floor(ref):
    """Error of the oracle's own values after rounding to bf16: (max, mean) of the metric."""
    rounded = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(ref.astype(np.float32))).astype(np.float64)
    mx, mean, _ = wl.rel_err_stats(rounded, ref)
    return mx, mean


def check_bf16(got, ref, what):
    mx, mean, _ = wl.rel_err_stats(got, ref)
    fmx, fmean = bf16_floor(ref)
    assert np.all(np.isfinite(got)), what
    assert mean <= 1.05 * fmean + 2e-5 and mx <= 2.0 ** -8 * 1.01, \
        "%s (bf16 out): max %.3e mean %.3e, rounding floor max %.3e mean %.3e" % (what, mx, mean, fmx, fmean)
