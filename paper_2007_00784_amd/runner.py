"""Drives a whole synthetic workload (a layer set) through the C-ABI library.

Holds device buffers and call order only: every arithmetic step is a library call.  Used by the
benchmark and by the full-size parity tests.
"""
import numpy as np
import torch

from . import kfac as K
from . import synthetic as S


class KfacRunner:
    def __init__(self, wl, device="cuda:0", n_updates=2, batch=None, layers=None, verbose=False):
        self.wl = wl
        self.dev = torch.device(device)
        self.N = wl.batch if batch is None else batch
        self.layer_ids = list(range(len(wl.layers))) if layers is None else list(layers)
        self.layers = [wl.layers[i] for i in self.layer_ids]
        self.n_updates = n_updates
        self.dt = torch.bfloat16 if wl.bf16 else torch.float32
        self.x, self.g = [], []          # [update][layer] device tensors
        self.gradw_master = []
        for u in range(n_updates):
            xs, gs = [], []
            for li in self.layer_ids:
                t = S.layer_inputs(wl, li, update=u, batch=self.N, want=("x", "g"))
                xs.append(self._up(t["x"]))
                gs.append(self._up(t["g"]))
                if verbose:
                    print("generated update %d layer %d" % (u, li), flush=True)
            self.x.append(xs)
            self.g.append(gs)
        # all gradients live in one flat buffer (and so do their masters), so that restoring them before an
        # in-place preconditioning is a single device copy
        gw = [S.layer_inputs(wl, li, batch=self.N, want=("gradw",))["gradw"] for li in self.layer_ids]
        offs = np.cumsum([0] + [(g.size + 63) // 64 * 64 for g in gw])
        self.gradw_master_flat = torch.zeros(int(offs[-1]), dtype=self.dt, device=self.dev)
        self.grad_flat = torch.zeros_like(self.gradw_master_flat)
        for j, g in enumerate(gw):
            view = self.gradw_master_flat[int(offs[j]):int(offs[j]) + g.size].view(g.shape)
            view.copy_(self._up(g))
            self.gradw_master.append(view)
        f32 = dict(dtype=torch.float32, device=self.dev)
        self.A = [torch.zeros((l.d_a, l.d_a), **f32) for l in self.layers]
        self.G = [torch.zeros((l.d_g, l.d_g), **f32) for l in self.layers]
        self.QA = [torch.zeros_like(a) for a in self.A]
        self.QG = [torch.zeros_like(g) for g in self.G]
        self.lamA = [torch.zeros(l.d_a, **f32) for l in self.layers]
        self.lamG = [torch.zeros(l.d_g, **f32) for l in self.layers]
        self.grad = [self.grad_flat[int(offs[j]):int(offs[j]) + g.size].view(g.shape) for j, g in enumerate(gw)]
        # every unfolded layer keeps its own patch slab, so all factor updates go out as one batch
        self.patches = [torch.empty((l.d_a - 1) * l.T * self.N, dtype=self.dt, device=self.dev) if l.needs_unfold else None
                        for l in self.layers]
        dims = [l.d_a for l in self.layers] + [l.d_g for l in self.layers]
        need = K.kfac_eig_workspace_bytes(dims)
        need = max(need, K.kfac_update_factors_workspace_bytes(self._factor_items(0, 0.0, sizing=True)))
        need = max(need, K.kfac_precondition_workspace_bytes([(l.d_a, l.d_g) for l in self.layers]))
        need = max(need, K.kfac_workspace_bytes(max(dims), 1, max(l.rows(self.N) for l in self.layers)))  # SYRK partials, precondition
        self.ws = torch.empty(need + 4096, dtype=torch.uint8, device=self.dev)
        self.stream = torch.cuda.current_stream(self.dev)
        self.ctx = K.kfac_create(self.dev.index or 0, self.stream.cuda_stream, self.ws)
        self.eig_info = None
        self._marshalled = {}    # item arrays of the batched calls, marshalled once per distinct argument set

    def _up(self, a):
        t = torch.from_numpy(np.ascontiguousarray(a)).to(self.dev)
        return t.to(torch.bfloat16) if self.wl.bf16 else t

    def close(self):
        torch.cuda.synchronize()
        if self.ctx is not None:
            K.kfac_destroy(self.ctx)
            self.ctx = None

    # ---- phases ----
    def _factor_items(self, upd, decay, sizing=False):
        N = self.N
        code = K.KFAC_BF16 if self.wl.bf16 else K.KFAC_F32
        items = []
        for i, l in enumerate(self.layers):
            R = N * l.T
            lay = K.KFAC_LAYOUT_RD if l.fc else K.KFAC_LAYOUT_NDT
            T = 1 if l.fc else l.T
            if sizing:
                src = g = FA = FG = None
            else:
                src = self.patches[i] if l.needs_unfold else self.x[upd][i]   # [N][C][H*W] is already the patch slab
                g, FA, FG = self.g[upd][i], self.A[i], self.G[i]
            items.append(dict(X=src, dtype=code, layout=lay, N=N, d=l.d_a - 1, T=T, append_ones=1, scale=1.0 / R,
                              decay=decay, F=FA))
            items.append(dict(X=g, dtype=code, layout=lay, N=N, d=l.d_g, T=T, append_ones=0, scale=1.0 / R,
                              decay=decay, F=FG))
        return items

    def update_factors(self, upd, decay, batched=True):
        idx = [i for i, l in enumerate(self.layers) if l.needs_unfold]
        if batched and idx:
            K.kfac_unfold_batched(self.ctx, [self.x[upd][i] for i in idx],
                                  [(self.layers[i].k, self.layers[i].k, self.layers[i].stride, self.layers[i].pad) for i in idx],
                                  [self.patches[i] for i in idx])
        else:
            for i in idx:
                l = self.layers[i]
                K.kfac_unfold(self.ctx, self.x[upd][i], l.k, l.k, l.stride, l.pad, self.patches[i])
        if batched:
            key = ("factors", upd, float(decay))
            if key not in self._marshalled:
                self._marshalled[key] = K.factor_items(self._factor_items(upd, decay))
            K.kfac_update_factors_batched(self.ctx, self._marshalled[key])
            return
        for it in self._factor_items(upd, decay):
            K.kfac_update_factors(self.ctx, it["X"], it["layout"], it["N"], it["d"], it["T"], it["append_ones"],
                                  it["scale"], it["decay"], it["F"], dtype=it["dtype"])

    def eig(self, **kw):
        self.eig_info = K.kfac_eig(self.ctx, self.A + self.G, self.QA + self.QG, self.lamA + self.lamG, **kw)
        return self.eig_info

    def restore_gradients(self):
        """Fresh gradients for the next in-place preconditioning (one device copy of the flat master buffer): what
        the backward pass of a training iteration delivers."""
        self.grad_flat.copy_(self.gradw_master_flat)

    def precondition(self, damping=None, kappa=None, lr=None, split_f16=None, restore=True):
        """In-place preconditioning of the gradients (restored from their masters first unless restore=False); with
        kappa and lr also the gradient scaling nu (left in self.nu, a device tensor).  split_f16 defaults to the
        workload's gradient type: bf16 gradients (rounding 4e-3) go through the split-fp16 GEMM chain (error 1e-6),
        fp32 ones through fp32."""
        gamma = self.wl.damping if damping is None else damping
        split = self.wl.bf16 if split_f16 is None else split_f16
        if restore:
            self.restore_gradients()
        key = ("precond", float(gamma), bool(split))
        if key not in self._marshalled:
            self._marshalled[key] = K.precond_items(self.QA, self.lamA, self.QG, self.lamG, gamma, self.grad, split_f16=split)
        if kappa is None:
            K.kfac_precondition_batched(self.ctx, items=self._marshalled[key])
        else:
            self.nu = torch.zeros(1, dtype=torch.float32, device=self.dev)
            K.kfac_precondition_batched_scaled(self.ctx, kappa=kappa, lr=lr, nu=self.nu, items=self._marshalled[key])

    # ---- the explicit-inverse method (Sec. II-C, Eq. (kfac-damped)): the paper's other way to the same step ----
    def invert_factors(self, damping=None):
        """(A + gamma I)^-1 and (G + gamma I)^-1 of every layer by blocked Cholesky (buffers allocated on first use)."""
        gamma = self.wl.damping if damping is None else damping
        if not hasattr(self, "Ainv"):
            self.Ainv = [torch.empty_like(a) for a in self.A]
            self.Ginv = [torch.empty_like(g) for g in self.G]
        K.kfac_invert_factors(self.ctx, self.A + self.G, gamma, self.Ainv + self.Ginv)

    def precondition_inverse(self, restore=True):
        """grad <- Ginv grad Ainv for every layer, in place."""
        if restore:
            self.restore_gradients()
        if "precond_inv" not in self._marshalled:
            self._marshalled["precond_inv"] = K.precond_inv_items(self.Ainv, self.Ginv, self.grad)
        K.kfac_precondition_inverse_batched(self.ctx, items=self._marshalled["precond_inv"])

    # ---- algorithmic work of one step (flops, bytes) ----
    def work(self):
        N = self.N
        esz = 2 if self.wl.bf16 else 4
        w = dict(syrk_flops=0.0, precond_flops=0.0, unfold_bytes=0.0, ema_bytes=0.0, sum_d3=0.0)
        for l in self.layers:
            R = N * l.T
            w["syrk_flops"] += R * (l.d_a * (l.d_a + 1.0) + l.d_g * (l.d_g + 1.0))
            w["precond_flops"] += 4.0 * l.d_a * l.d_g * (l.d_a + l.d_g)
            if l.needs_unfold:
                w["unfold_bytes"] += esz * (N * l.c_in * l.h_in * l.h_in + R * (l.d_a - 1.0))
            w["ema_bytes"] += 8.0 * (l.d_a ** 2 + l.d_g ** 2)
            w["sum_d3"] += float(l.d_a) ** 3 + float(l.d_g) ** 3
        return w
