"""Drives one Symi iteration through the C ABI (via the thin binding) on cuda:0.

Plumbing only: allocates tensors with torch, draws inputs from `workloads`, calls the
library in the order of paper Fig. 5 and hands back every buffer.  No arithmetic of the
method happens here (slot weights are materialised from class weights by indexing).
"""
from types import SimpleNamespace

import numpy as np
import torch

import paper_2504_19925_amd as symi
import workloads as wl

HP = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, grad_scale=1.0, step=1)


def make_cfg(c: wl.Config, shard=0, renorm=1):
    return symi.SymiCfg.make(c.T, c.E, c.k, c.d, c.f, c.S_tot, c.N, shard, c.dtype, renorm)


def make_ctx(c: wl.Config, shard=0, renorm=1, flags=0):
    """A library context (symi_create) for workload c on the current device."""
    return symi.symi_create(make_cfg(c, shard, renorm), flags)


def make_adam(**kw):
    hp = dict(HP)
    hp.update(kw)
    # the C ABI takes fp32 hyper-parameters: both sides get exactly those values
    hp = {k: (float(np.float32(v)) if k != "step" else int(v)) for k, v in hp.items()}
    return symi.SymiAdam(hp["lr"], hp["beta1"], hp["beta2"], hp["eps"], hp["weight_decay"],
                         hp["grad_scale"], hp["step"]), hp


class State:
    """Buffers that persist across iterations of one config (all on the GPU)."""

    def __init__(self, c: wl.Config, dev="cuda", shard=0, renorm=1, weights=None, flags=0,
                 all_shards=False):
        """shard: the optimizer partition this state's context (and .master/.m/.v) belongs to.
        all_shards: also hold the other N-1 partitions (contexts and Adam state), so that
        optimizer() rewrites the whole of every slot, as the N ranks of the method do."""
        self.c, self.dev = c, dev
        self.active_grads = False   # True: the *_active pair (classes without rows are skipped)
        self.ctx = make_ctx(c, shard, renorm, flags)
        self.cfg = self.ctx.cfg
        dt = self.cfg.torch_dtype
        i32 = dict(dtype=torch.int32, device=dev)
        E, S, A, T, d, f = c.E, c.S_tot, c.A, c.T, c.d, c.f
        self.W1c, self.W2c = weights if weights is not None else wl.make_class_weights(c, dev)
        self.hist_prev = torch.zeros(E, **i32)          # no popularity yet: uniform placement
        self.counts = torch.empty(E, **i32)
        self.placement = torch.empty(S, **i32)
        self.first_slot = torch.empty(E + 1, **i32)
        self.counts_next = torch.empty(E, **i32)
        self.placement_next = torch.empty(S, **i32)
        self.first_slot_next = torch.empty(E + 1, **i32)
        self.idx = torch.empty(T, c.k, **i32)
        self.gate = torch.empty(T, c.k, dtype=torch.float32, device=dev)
        self.hist = torch.empty(E, **i32)
        self.row_of_assign = torch.empty(A, **i32)
        self.assign_of_row = torch.empty(A, **i32)
        self.slot_offsets = torch.empty(S + 1, **i32)
        self.ws = torch.empty(symi.symi_workspace_bytes(self.cfg), dtype=torch.uint8, device=dev)
        mk = lambda *s: torch.empty(*s, dtype=dt, device=dev)
        self.Xp, self.Yp, self.dYp, self.dXp = mk(A, d), mk(A, d), mk(A, d), mk(A, d)
        self.UV, self.H = mk(A, 2 * f), mk(A, f)
        self.Y, self.dX = mk(T, d), mk(T, d)
        self.dgate = torch.empty(T, c.k, dtype=torch.float32, device=dev)
        self.dlogits = torch.empty(T, E, dtype=torch.float32, device=dev)
        self.dW1 = torch.empty(E, 2 * f, d, dtype=torch.float32, device=dev)
        self.dW2 = torch.empty(E, d, f, dtype=torch.float32, device=dev)
        self.W1s = torch.empty(S, 2 * f, d, dtype=dt, device=dev)
        self.W2s = torch.empty(S, d, f, dtype=dt, device=dev)
        # this partition's optimizer state: master weights start as the class weights
        per = c.P_e // c.N
        self.opt = {}     # shard -> (context, master, m, v)
        for n in (range(c.N) if all_shards else [shard]):
            lo = n * per
            n1 = 2 * f * d
            parts = []
            if lo < n1:
                parts.append(self.W1c.reshape(E, -1)[:, lo:min(lo + per, n1)])
            if lo + per > n1:
                parts.append(self.W2c.reshape(E, -1)[:, max(lo - n1, 0):lo + per - n1])
            master = torch.cat(parts, dim=1).to(torch.float32).contiguous()
            ctx_n = self.ctx if n == shard else make_ctx(c, n, renorm, symi.CTX_NO_OVERLAP)
            self.opt[n] = (ctx_n, master, torch.zeros_like(master), torch.zeros_like(master))
        _, self.master, self.m, self.v = self.opt[shard]

    def place_current(self):
        """Placement of the coming iteration from the previous iteration's popularity,
        and slot weights materialised from the class weights (every replica of a class
        holds the same weights)."""
        symi.symi_place(self.ctx, self.hist_prev, self.counts, self.placement, self.first_slot)
        pl = self.placement.long()
        torch.index_select(self.W1c, 0, pl, out=self.W1s)
        torch.index_select(self.W2c, 0, pl, out=self.W2s)

    def forward(self, X, logits, slot_cap=None):
        """slot_cap: rows a slot may take (capacity-limited dispatch); None = dropless."""
        s, ctx = self, self.ctx
        symi.symi_route(ctx, logits, s.idx, s.gate, s.hist)
        if slot_cap is None:
            symi.symi_dispatch(ctx, X, s.idx, s.hist, s.counts, s.first_slot, s.row_of_assign,
                               s.assign_of_row, s.slot_offsets, s.Xp, s.ws)
        else:
            symi.symi_dispatch_capacity(ctx, slot_cap, X, s.idx, s.hist, s.counts, s.first_slot,
                                        s.row_of_assign, s.assign_of_row, s.slot_offsets, s.Xp, s.ws)
        symi.symi_expert_fwd(ctx, s.Xp, s.slot_offsets, s.W1s, s.W2s, s.UV, s.H, s.Yp, s.ws)
        symi.symi_combine(ctx, s.Yp, s.row_of_assign, s.gate, s.Y)

    def backward(self, dY, logits):
        s, ctx = self, self.ctx
        symi.symi_combine_bwd(ctx, dY, s.Yp, s.row_of_assign, s.gate, s.dYp, s.dgate)
        bwd = symi.symi_expert_bwd_active if s.active_grads else symi.symi_expert_bwd
        bwd(ctx, s.dYp, s.Xp, s.UV, s.H, s.slot_offsets, s.first_slot, s.W1s, s.W2s,
            s.dXp, s.dW1, s.dW2, s.ws)
        symi.symi_dispatch_bwd(ctx, s.dXp, s.row_of_assign, s.dX)
        symi.symi_route_bwd(ctx, logits, s.idx, s.gate, s.dgate, s.dlogits)

    def optimizer(self, adam, shards=None):
        """Next placement, then Adam + replica write for the held partitions (or `shards`)."""
        s = self
        symi.symi_place(s.ctx, s.hist, s.counts_next, s.placement_next, s.first_slot_next)
        for n in (s.opt if shards is None else shards):
            ctx, master, m, v = s.opt[n]
            if s.active_grads:   # gradients of classes without rows were not written: do not read them
                symi.symi_adam_to_replicas_active(ctx, adam, s.dW1, s.dW2, master, m, v,
                                                  s.slot_offsets, s.first_slot, s.first_slot_next,
                                                  s.W1s, s.W2s)
            else:
                symi.symi_adam_to_replicas(ctx, adam, s.dW1, s.dW2, master, m, v, s.first_slot_next,
                                           s.W1s, s.W2s)

    def advance(self):
        """The placement computed by optimizer() becomes the one the next iteration dispatches
        with (the two sets of placement buffers swap roles)."""
        s = self
        s.counts, s.counts_next = s.counts_next, s.counts
        s.first_slot, s.first_slot_next = s.first_slot_next, s.first_slot
        s.placement, s.placement_next = s.placement_next, s.placement


def draw_inputs(c: wl.Config, it=0, dev="cuda"):
    X = wl.make_tokens(c, it, dev)
    logits = wl.make_logits(c, it, dev, tokens=X)
    dY = wl.make_upstream_grad(c, it, dev)
    return X, logits, dY


def npf(t):
    """GPU/CPU tensor -> numpy (bf16 widened to fp32, exact)."""
    t = t.detach()
    if t.dtype == torch.bfloat16:
        t = t.to(torch.float32)
    return t.cpu().numpy()


class LazyWeights:
    """Per-class view of a [E, r, c] GPU tensor for the oracle: converts one class at a
    time so that full-size configs never hold an fp64 copy of every class on the host."""

    def __init__(self, t, rows=None, cols=None):
        self.t, self.rows, self.cols = t, rows, cols
        r = t.shape[1] if rows is None else len(rows)
        cdim = t.shape[2] if cols is None else len(cols)
        self.shape = (t.shape[0], r, cdim)

    def _cls(self, e):
        x = self.t[e]
        if self.rows is not None:
            x = x[self.rows]
        if self.cols is not None:
            x = x[:, self.cols]
        return x.to(torch.float32).cpu().numpy()

    def __getitem__(self, key):
        if isinstance(key, tuple):
            return self._cls(int(key[0]))[key[1:] if len(key) > 2 else key[1]]
        return self._cls(int(key))


def sync():
    torch.cuda.synchronize()
