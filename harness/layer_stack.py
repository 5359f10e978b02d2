"""A decode step through a stack of decoder layers' linear projections, for one HIP graph.

Rollout decode dominates the run time of the paper's system (Sec. 1, Sec. 3), and what a rollout
engine launches per token step is, per layer, the block's projections one after the other, all on
the same token -> adapter map (Sec. 4.5: many tasks' adapters on one frozen base model).  This
module builds that sequence for L layers out of the library's calls:

    q, k, v = fwd_multi(x)            one pass over x, three projections, one table of adapters
    o       = fwd(q)                  (attention itself is not part of this path: q stands in for it)
    h       = bf16(x + o)
    g, up   = fwd_multi(h)            gate and up projections
    m       = bf16(bf16(silu(g)) * up)
    dn      = fwd(m)                  down projection
    x'      = bf16(h + dn)

Every projection has its own frozen weight, packed once for the decode kernel, and its own rank-r
adapters for every task, registered once in adapter tables; the elementwise glue between the calls
is plain torch (a handful of small kernels, captured with the rest).  Nothing here computes any of
the layer's arithmetic: it only wires buffers to calls.  Used by bench.py (timing, full sizes) and
by the GPU tests (every call of the stack against the oracle, small sizes).
"""
import numpy as np


def _normal(shape, std, gen, torch):
    t = torch.empty(shape, dtype=torch.float32, device="cuda")
    t.normal_(0.0, std, generator=gen)
    return t.to(torch.bfloat16)


class Projection:
    """One frozen weight with its adapters (torch layout: W[d_out, d_in], A_t[r, d_in], B_t[d_out, r])."""

    def __init__(self, K, N, ranks, gen, torch, w_gain, b_gain):
        self.K, self.N = K, N
        self.W = _normal((N, K), w_gain * K ** -0.5, gen, torch)
        self.A = [_normal((int(r), K), K ** -0.5, gen, torch) for r in ranks]
        self.B = [_normal((N, int(r)), b_gain * float(r) ** -0.5, gen, torch) for r in ranks]
        self.Wp = None


class Group:
    """Projections that read the same input in one call (one adapter table of len(projs) projections)."""

    def __init__(self, name, x, projs, outs, stack):
        api, torch = stack.api, stack.torch
        self.name, self.x, self.projs, self.outs = name, x, projs, outs
        self.table = api.marlaas_adapter_table_create(stack.ctx, stack.n, len(projs), int(max(stack.ranks)))
        self.descs = []
        for p, pr in enumerate(projs):
            for t in range(stack.n):
                api.marlaas_adapter_table_update(stack.ctx, self.table, p, t, pr.A[t], pr.B[t], int(stack.ranks[t]),
                                                 float(stack.scales[t]))
            if stack.packed:
                pr.Wp = api.marlaas_pack_weight(stack.ctx, pr.W, 1, 0)
            self.descs.append(api.LoraDesc(x, pr.W, None, None, None, None, stack.segmap, layout=1,
                                           out_dtype=torch.bfloat16, table=self.table, proj=p, W_packed_fwd=pr.Wp))

    def workspace_bytes(self, api):
        if len(self.descs) > 1:
            return api.marlaas_workspace_bytes_multi(self.descs)
        return api.marlaas_workspace_bytes(self.descs[0], False)

    def run(self, api, ctx):
        if len(self.descs) > 1:
            api.marlaas_lora_fwd_multi(ctx, self.descs, self.outs)
        else:
            api.marlaas_lora_fwd(ctx, self.descs[0], self.outs[0])


class DecodeStack:
    def __init__(self, api, torch, ctx, ids, T, d, d_kv, d_ff, L, ranks, scales, seed=0, packed=True, w_gain=0.5, b_gain=0.25):
        """ids: int32 device tensor [T] (token -> adapter, -1: none); ranks / scales per adapter.
        w_gain and b_gain scale the init of the weights and of the B factors (against the single
        layer's recipe) so that activations stay O(1) through the residual stack."""
        self.api, self.torch, self.ctx = api, torch, ctx
        self.T, self.d, self.d_kv, self.d_ff, self.L = T, d, d_kv, d_ff, L
        self.ranks, self.scales, self.n, self.packed = list(ranks), list(scales), len(ranks), packed
        self.segmap = api.marlaas_segmap_build(ctx, ids, self.n)
        gen = torch.Generator(device="cuda")
        gen.manual_seed(1000 + seed)
        bf = dict(dtype=torch.bfloat16, device="cuda")
        self.x0 = _normal((T, d), 1.0, gen, torch)
        self.layers = []
        x = self.x0
        for _ in range(L):
            buf = dict(q=torch.empty((T, d), **bf), k=torch.empty((T, d_kv), **bf), v=torch.empty((T, d_kv), **bf),
                       o=torch.empty((T, d), **bf), h=torch.empty((T, d), **bf), g=torch.empty((T, d_ff), **bf),
                       up=torch.empty((T, d_ff), **bf), sg=torch.empty((T, d_ff), **bf), m=torch.empty((T, d_ff), **bf),
                       dn=torch.empty((T, d), **bf), x_out=torch.empty((T, d), **bf))
            mk = lambda K, N: Projection(K, N, self.ranks, gen, torch, w_gain, b_gain)
            groups = [Group("qkv", x, [mk(d, d), mk(d, d_kv), mk(d, d_kv)], [buf["q"], buf["k"], buf["v"]], self),
                      Group("o", buf["q"], [mk(d, d)], [buf["o"]], self),
                      Group("gate_up", buf["h"], [mk(d, d_ff), mk(d, d_ff)], [buf["g"], buf["up"]], self),
                      Group("down", buf["m"], [mk(d_ff, d)], [buf["dn"]], self)]
            self.layers.append(dict(x_in=x, buf=buf, groups=groups))
            x = buf["x_out"]
        self.out = x
        need = max(g.workspace_bytes(api) for lay in self.layers for g in lay["groups"])
        self.ws = torch.empty(max(int(need), 256), dtype=torch.uint8, device="cuda")
        api.marlaas_set_workspace(ctx, self.ws)
        torch.cuda.synchronize()

    def step(self):
        """One token step: every layer's four calls and the glue, enqueued on the current stream."""
        api, torch, ctx = self.api, self.torch, self.ctx
        for lay in self.layers:
            b, (qkv, o, gate_up, down) = lay["buf"], lay["groups"]
            qkv.run(api, ctx)
            o.run(api, ctx)
            torch.add(lay["x_in"], b["o"], out=b["h"])
            gate_up.run(api, ctx)
            torch.ops.aten.silu.out(b["g"], out=b["sg"])
            torch.mul(b["sg"], b["up"], out=b["m"])
            down.run(api, ctx)
            torch.add(b["h"], b["dn"], out=b["x_out"])

    def capture(self):
        """The step as one HIP graph (the passes allocate nothing, so a first call may be captured)."""
        torch = self.torch
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.step()
        return graph

    def weight_bytes(self):
        """Bytes of frozen weights one step has to read (the dominant algorithmic traffic)."""
        return sum(2 * pr.K * pr.N for lay in self.layers for g in lay["groups"] for pr in g.projs)

    def algorithmic_bytes(self, present):
        """Minimum bytes of one step: every weight once, every call's input and outputs once, the
        factors of the adapters that have tokens (present: boolean per adapter)."""
        rsum = float(np.sum(np.asarray(self.ranks)[np.asarray(present)]))
        total = 0.0
        for lay in self.layers:
            for g in lay["groups"]:
                total += 2.0 * self.T * g.projs[0].K
                for pr in g.projs:
                    total += 2.0 * pr.K * pr.N + 2.0 * self.T * pr.N + 2.0 * rsum * (pr.K + pr.N)
        return total
