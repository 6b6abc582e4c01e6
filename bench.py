"""Benchmark of the decomposed-layer forward + backward path on one MI355X.  Prints ONE JSON line.

Headline workload (synthetic, seeded): the decomposed linear layers of a 12-layer transformer encoder,
hidden 1024, FFN 4096, 8192 tokens (batch 16 x sequence 512), bf16.  Per layer: the query / key / value
projections as one grouped call on the shared input (1024 -> 3 x 1024), the attention output projection
(1024 -> 1024), the FFN up-projection (1024 -> 4096, GELU folded into the call) and down-projection
(4096 -> 1024); every weight is an SVD pair at the quantized rank 256; the freeze mask of step s is
Algorithm 2's mask for epoch s for every layer (first factors frozen on even steps, second factors on odd
steps).  One step = forward through all 12 layers, then backward.  The attention itself (softmax(QK^T)V),
layer norms and residual additions are unchanged by the method and are not run: each layer's attention
output and the gradient reaching its Q / K / V outputs are fixed synthetic tensors of the right shape, so
every decomposed-layer kernel runs at its real shape on its own buffers.

`value` is the algorithmic TFLOP/s of the decomposed layers (FLOPs as masked by freezing), all inputs
resident in HBM before the timed region, the K timed steps replayed from two captured HIP graphs (even /
odd mask) after each replay was checked bit for bit against eager launches.  Beside it: tokens/s, the
fraction of the step's binding roof (per layer pass max(flops / MFMA peak, algorithmic bytes / HBM peak),
summed), the roofline of the product kernel with the largest share of the step (timed with HIP events in
an eager pass over the same K steps), peaks measured in the same run (register-only MFMA loop, plain
stream kernel), the undecomposed encoder and the raw-rank / unfrozen pair stacks, the other workloads
(12-block FFN stack at rank 192; one 4096 x 4096 layer at ranks 256 / 257 / 512 / 1024; four Tucker 3x3
stages at N = 128) each with time, TFLOP/s and binding-roof fraction, and the CPU oracle on a bounded
sample.  Other modes (see --help) print their own single JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

T_TOKENS, D_MODEL, D_FF, N_BLOCKS = 8192, 768, 3072, 12            # FFN-stack workload (rank 192)
ENC_T, ENC_D, ENC_FF, ENC_LAYERS, ENC_RANK = 8192, 1024, 4096, 12, 256   # encoder workload (headline)
HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0


def layer_flops(T, n_in, n_out, r, mask, want_dx=True):
    fwd = 2 * T * r * (n_in + n_out)
    bwd = 2 * T * r * n_out + (2 * T * r * n_in if want_dx else 0)
    bwd += 0 if mask & 2 else 2 * T * r * n_out
    bwd += 0 if mask & 1 else 2 * T * r * n_in
    return fwd, bwd


class Stack:
    """Buffers and factors of the 12-block stack; fwd/bwd through the library only.  deferred=True runs the
    backward in two parts (data gradients per block, then each of the two layer shapes' weight gradients
    for all blocks in one call); the per-block tensors are slices of stacks over the blocks."""

    def __init__(self, lrd, torch, np, si, factorize, rank, seed_stream, true_svd=True, deferred=False):
        self.lrd, self.torch, self.deferred = lrd, torch, deferred
        dev = "cuda"
        bf = torch.bfloat16
        rng = si.rng_for(2, seed_stream)
        self.r = rank
        self.layers = []
        T, NB = T_TOKENS, N_BLOCKS

        def to_dev(a):
            bits = si.bf16_bits(a).view(np.int16)
            return torch.from_numpy(bits).to(dev).view(bf).reshape(a.shape)

        def empty(*shape, dt=bf):
            return torch.empty(shape, dtype=dt, device=dev)

        dims = ((D_MODEL, D_FF), (D_FF, D_MODEL))
        self.st = [dict(H=empty(NB, T, rank), dH=empty(NB, T, rank), dU=empty(NB, n_out, rank, dt=torch.float32),
                        dV=empty(NB, rank, n_in, dt=torch.float32)) for (n_in, n_out) in dims]
        for b in range(NB):
            blk = []
            for i, (n_in, n_out) in enumerate(dims):
                if true_svd:
                    W = si.linear_weight(n_out, n_in, rng)
                    U, V, _ = factorize.svd_factors(W, rank)
                else:
                    U, V = si.direct_factors(n_out, n_in, rank, rng)
                s = self.st[i]
                blk.append(dict(n_in=n_in, n_out=n_out, U=to_dev(U), V=to_dev(V), H=s["H"][b], dH=s["dH"][b], dU=s["dU"][b],
                                dV=s["dV"][b]))
            self.layers.append(blk)
        # G[b] is the gradient entering block b's second layer; the stack's output is G[NB - 1] (loss 0.5 ||Y||^2)
        self.Xs, self.G = empty(NB, T, D_MODEL), empty(NB, T, D_MODEL)
        self.Xs[0].copy_(to_dev(si.gaussian((T, D_MODEL), rng)))
        self.X = [self.Xs[b] for b in range(NB)] + [self.G[NB - 1]]
        self.Zs, self.As, self.gZs = empty(NB, T, D_FF), empty(NB, T, D_FF), empty(NB, T, D_FF)
        self.Z, self.A = [self.Zs[b] for b in range(NB)], [self.As[b] for b in range(NB)]
        self.gZ = self.gZs[0]
        self.gX = [self.G[b & 1] for b in range(2)]      # (used by callers that run their own per-block backward)
        nbytes = max(lrd.linear_workspace_bytes(T, D_MODEL, D_FF, rank, lrd.BF16, 0),
                     lrd.linear_workspace_bytes(T, D_FF, D_MODEL, rank, lrd.BF16, 0),
                     lrd.linear_wgrad_batched_workspace_bytes(NB, T, D_MODEL, D_FF, rank, lrd.BF16, 0),
                     lrd.linear_wgrad_batched_workspace_bytes(NB, T, D_FF, D_MODEL, rank, lrd.BF16, 0))
        self.ws = torch.empty(nbytes + 256, dtype=torch.uint8, device=dev)

    def forward(self):
        lrd = self.lrd
        for b, (l1, l2) in enumerate(self.layers):
            lrd.linear_fwd_act(self.X[b], l1["V"], l1["U"], None, self.Z[b], self.A[b], l1["H"], lrd.ACT_GELU, self.ws)
            lrd.linear_fwd(self.A[b], l2["V"], l2["U"], None, self.X[b + 1], l2["H"], self.ws)

    def backward(self, mask):
        """Loss 0.5 ||Y||^2: the gradient entering the last block is the stack's output."""
        lrd = self.lrd
        if self.deferred:
            for b in reversed(range(N_BLOCKS)):
                l1, l2 = self.layers[b]
                lrd.linear_bwd_data(self.G[b], l2["V"], l2["U"], self.gZs[b], l2["dH"], self.Z[b], lrd.ACT_GELU, self.ws)
                lrd.linear_bwd_data(self.gZs[b], l1["V"], l1["U"], self.G[b - 1] if b > 0 else None, l1["dH"], None, lrd.ACT_NONE, self.ws)
            tu, tv = not mask & 2, not mask & 1
            for s, dY, X in ((self.st[1], self.G, self.As), (self.st[0], self.gZs, self.Xs)):
                lrd.linear_wgrad_batched(dY if tu else None, s["H"] if tu else None, s["dH"] if tv else None, X if tv else None,
                                         s["dV"], s["dU"], mask, self.ws)
            return
        # one call per layer; the gradient buffers alternate (the stack's output in G[NB - 1] is read by the first call only)
        g = self.X[N_BLOCKS]
        for b in reversed(range(N_BLOCKS)):
            l1, l2 = self.layers[b]
            out = self.G[b - 1] if b > 0 else None
            lrd.linear_bwd_act(g, self.A[b], l2["H"], l2["V"], l2["U"], self.gZ, l2["dV"], l2["dU"], None, mask,
                               self.Z[b], lrd.ACT_GELU, self.ws)
            lrd.linear_bwd(self.gZ, self.X[b], l1["H"], l1["V"], l1["U"], out, l1["dV"], l1["dU"], None, mask, self.ws)
            g = out

    def step(self, mask):
        self.forward()
        self.backward(mask)

    def flops(self, mask):
        tot = 0
        for b in range(N_BLOCKS):
            f1, b1 = layer_flops(T_TOKENS, D_MODEL, D_FF, self.r, mask, want_dx=b > 0)
            f2, b2 = layer_flops(T_TOKENS, D_FF, D_MODEL, self.r, mask)
            tot += f1 + b1 + f2 + b2
        return tot


class DenseStack:
    def __init__(self, lrd, torch, np, si):
        self.lrd = lrd
        dev, bf = "cuda", torch.bfloat16
        rng = si.rng_for(2, 7)
        T = T_TOKENS

        def to_dev(a):
            bits = si.bf16_bits(a).view(np.int16)
            return torch.from_numpy(bits).to(dev).view(bf).reshape(a.shape)

        self.W = [(to_dev(si.linear_weight(D_FF, D_MODEL, rng)), to_dev(si.linear_weight(D_MODEL, D_FF, rng)))
                  for _ in range(N_BLOCKS)]
        self.dW = (torch.empty((D_FF, D_MODEL), dtype=torch.float32, device=dev),
                   torch.empty((D_MODEL, D_FF), dtype=torch.float32, device=dev))
        self.X = [to_dev(si.gaussian((T, D_MODEL), rng))] + [torch.empty((T, D_MODEL), dtype=bf, device=dev) for _ in range(N_BLOCKS)]
        self.Z = [torch.empty((T, D_FF), dtype=bf, device=dev) for _ in range(N_BLOCKS)]
        self.A = [torch.empty((T, D_FF), dtype=bf, device=dev) for _ in range(N_BLOCKS)]
        self.gX = [torch.empty((T, D_MODEL), dtype=bf, device=dev) for _ in range(2)]
        self.gA = torch.empty((T, D_FF), dtype=bf, device=dev)
        self.gZ = torch.empty((T, D_FF), dtype=bf, device=dev)
        nbytes = max(lrd.dense_linear_workspace_bytes(T, D_MODEL, D_FF, lrd.BF16),
                     lrd.dense_linear_workspace_bytes(T, D_FF, D_MODEL, lrd.BF16))
        self.ws = torch.empty(nbytes + 256, dtype=torch.uint8, device=dev)

    def step(self, mask=0):
        lrd = self.lrd
        for b, (w1, w2) in enumerate(self.W):
            lrd.dense_linear_fwd(self.X[b], w1, None, self.Z[b], self.ws)
            lrd.gelu_fwd(self.Z[b], self.A[b])
            lrd.dense_linear_fwd(self.A[b], w2, None, self.X[b + 1], self.ws)
        g = self.X[N_BLOCKS]
        for b in reversed(range(N_BLOCKS)):
            w1, w2 = self.W[b]
            out = self.gX[b & 1]
            lrd.dense_linear_bwd(g, self.A[b], w2, self.gA, self.dW[1], self.ws)
            lrd.gelu_bwd(self.gA, self.Z[b], self.gZ)
            lrd.dense_linear_bwd(self.gZ, self.X[b], w1, out if b > 0 else None, self.dW[0], self.ws)
            g = out


def linear_bytes(T, n_in, n_out, r, mask, want_dx=True, act_out=False, act_in=False):
    """Algorithmic bytes of one decomposed bf16 layer, (forward, backward): activations and factors
    read once, results written once; the rank-r intermediate H is written by the forward only when the
    backward will need it (second factor trainable) and dH never leaves the chip; fp32 gradients of
    the trainable factors written once.  act_out: the forward also writes the activation of its result
    (folded GELU); act_in: the backward also reads the pre-activation of its input."""
    e = 2
    fwd = e * (T * n_in + T * n_out + r * (n_in + n_out))
    if not mask & 2:
        fwd += e * T * r
    if act_out:
        fwd += e * T * n_out
    bwd = e * T * n_out + e * r * (n_in + n_out)
    if want_dx:
        bwd += e * T * n_in
    if act_in and want_dx:
        bwd += e * T * n_in
    if not mask & 1:
        bwd += e * T * n_in + 4 * r * n_in
    if not mask & 2:
        bwd += e * T * r + 4 * r * n_out
    return fwd, bwd


def roof_us(flops, nbytes):
    """Lower bound of a pass in microseconds and which roof binds it."""
    t_mfma, t_hbm = flops / (MFMA_BF16_PEAK_TFLOPS * 1e12) * 1e6, nbytes / (HBM_PEAK_GBS * 1e9) * 1e6
    return max(t_mfma, t_hbm), ("mfma" if t_mfma >= t_hbm else "hbm")


class Encoder:
    """The decomposed linears of a 12-layer encoder (hidden 1024, FFN 4096), rank r; fwd/bwd through the library only.

    Every per-layer tensor is a slice of a stack over the layers.  deferred=True runs the backward in
    two parts: data gradients layer by layer, then the weight gradients of all layers of one shape in
    one call each (the stacks hand that call its operands at a fixed stride)."""

    def __init__(self, lrd, torch, np, si, rank, seed_stream, layers=ENC_LAYERS, grouped=True, deferred=False):
        self.lrd, self.torch, self.r, self.n_layers, self.grouped = lrd, torch, rank, layers, grouped
        self.deferred = deferred and grouped
        dev, bf = "cuda", torch.bfloat16
        rng = si.rng_for(5, seed_stream)
        T, d, ff, L = ENC_T, ENC_D, ENC_FF, layers

        def to_dev(a):
            bits = si.bf16_bits(a).view(np.int16)
            return torch.from_numpy(bits).to(dev).view(bf).reshape(a.shape)

        def empty(*shape, dt=bf):
            return torch.empty(shape, dtype=dt, device=dev)

        def stack(n_out, n_in):
            return dict(H=empty(L, T, rank), dH=empty(L, T, rank), dU=empty(L, n_out, rank, dt=torch.float32),
                        dV=empty(L, rank, n_in, dt=torch.float32))

        self.st = dict(o=stack(d, d), up=stack(ff, d), dn=stack(d, ff),
                       qkv=dict(H=empty(L, T, 3 * rank), dH=empty(L, T, 3 * rank), dU=empty(L, 3, d, rank, dt=torch.float32),
                                dU_by_member=empty(3, L, d, rank, dt=torch.float32), dV=empty(L, 3 * rank, d, dt=torch.float32)))
        # stand-ins for what the (unchanged, not run) attention hands to and receives from these layers
        self.attn, self.dqkv = empty(L, T, d), empty(L, 3, T, d)
        self.Xo, self.Z, self.A = empty(L, T, d), empty(L, T, ff), empty(L, T, ff)
        # gradient stacks: G[l] enters layer l's second FFN linear (G[L-1] is the stack's own output)
        self.G, self.gZ, self.gXo, self.gAttn = empty(L, T, d), empty(L, T, ff), empty(L, T, d), empty(T, d)
        self.Xs = empty(L, T, d)
        self.Xs[0].copy_(to_dev(si.gaussian((T, d), rng)))
        self.X = [self.Xs[l] for l in range(L)] + [self.G[L - 1]]

        def pair(name, l, n_out, n_in):
            U, V = si.direct_factors(n_out, n_in, rank, rng)
            return dict(U=to_dev(U), V=to_dev(V), H=self.st[name]["H"][l], dH=self.st[name]["dH"][l], dU=self.st[name]["dU"][l],
                        dV=self.st[name]["dV"][l])

        self.layers = []
        for l in range(L):
            qkv = [si.direct_factors(d, d, rank, rng) for _ in range(3)]
            q = self.st["qkv"]
            Lr = dict(o=pair("o", l, d, d), up=pair("up", l, ff, d), dn=pair("dn", l, d, ff),
                      qkv=dict(U=to_dev(np.stack([u for u, _ in qkv])), V=to_dev(np.concatenate([v for _, v in qkv], axis=0)),
                               H=q["H"][l], dH=q["dH"][l], dU=q["dU"][l], dV=q["dV"][l],
                               Y=empty(3, T, d), Hs=None if grouped else [empty(T, rank) for _ in range(3)]),
                      attn=self.attn[l], dqkv=self.dqkv[l], Xo=self.Xo[l], Z=self.Z[l], A=self.A[l])
            self.attn[l].copy_(to_dev(si.gaussian((T, d), rng)))
            self.dqkv[l].copy_(to_dev(si.gaussian((3, T, d), rng, 1e-2)))
            self.layers.append(Lr)
        self.gQ = None if grouped else [empty(T, d) for _ in range(3)]
        nbytes = max(lrd.linear_workspace_bytes(T, d, d, rank, lrd.BF16, 0), lrd.linear_workspace_bytes(T, d, ff, rank, lrd.BF16, 0),
                     lrd.linear_workspace_bytes(T, ff, d, rank, lrd.BF16, 0),
                     lrd.linear_group_workspace_bytes(T, d, d, rank, 3, lrd.BF16, 0),
                     lrd.linear_wgrad_batched_workspace_bytes(L, T, d, d, 3 * rank, lrd.BF16, 0),
                     lrd.linear_wgrad_batched_workspace_bytes(L, T, d, ff, rank, lrd.BF16, 0),
                     lrd.linear_wgrad_batched_workspace_bytes(L, T, ff, d, rank, lrd.BF16, 0))
        self.ws = torch.empty(nbytes + 256, dtype=torch.uint8, device=dev)

    def forward(self):
        lrd = self.lrd
        for l, L in enumerate(self.layers):
            q, o, up, dn = L["qkv"], L["o"], L["up"], L["dn"]
            if self.grouped:
                lrd.linear_group_fwd(self.X[l], q["V"], q["U"], None, q["Y"], q["H"], self.ws)
            else:
                for g in range(3):
                    lrd.linear_fwd(self.X[l], q["V"][g * self.r:(g + 1) * self.r], q["U"][g], None, q["Y"][g], q["Hs"][g], self.ws)
            lrd.linear_fwd(L["attn"], o["V"], o["U"], None, L["Xo"], o["H"], self.ws)
            lrd.linear_fwd_act(L["Xo"], up["V"], up["U"], None, L["Z"], L["A"], up["H"], lrd.ACT_GELU, self.ws)
            lrd.linear_fwd(L["A"], dn["V"], dn["U"], None, self.X[l + 1], dn["H"], self.ws)

    def backward(self, mask):
        """Loss 0.5 ||X_last||^2: the gradient entering the last layer is the stack's output."""
        if self.deferred:
            return self.backward_deferred(mask)
        lrd = self.lrd
        for l in reversed(range(self.n_layers)):
            L = self.layers[l]
            q, o, up, dn = L["qkv"], L["o"], L["up"], L["dn"]
            g, out = self.G[l], (self.G[l - 1] if l > 0 else None)
            lrd.linear_bwd_act(g, L["A"], dn["H"], dn["V"], dn["U"], self.gZ[l], dn["dV"], dn["dU"], None, mask, L["Z"], lrd.ACT_GELU, self.ws)
            lrd.linear_bwd(self.gZ[l], L["Xo"], up["H"], up["V"], up["U"], self.gXo[l], up["dV"], up["dU"], None, mask, self.ws)
            lrd.linear_bwd(self.gXo[l], L["attn"], o["H"], o["V"], o["U"], self.gAttn, o["dV"], o["dU"], None, mask, self.ws)
            if self.grouped:
                lrd.linear_group_bwd(L["dqkv"], self.X[l], q["H"], q["V"], q["U"], out, q["dV"], q["dU"], None, mask, self.ws)
            else:
                # three separate layers; their input gradients are added afterwards (glue, not the library's)
                for i in range(3):
                    lrd.linear_bwd(L["dqkv"][i], self.X[l], q["Hs"][i], q["V"][i * self.r:(i + 1) * self.r], q["U"][i],
                                   self.gQ[i] if l > 0 else None, q["dV"][i * self.r:(i + 1) * self.r], q["dU"][i], None, mask, self.ws)
                if l > 0:
                    self.torch.add(self.gQ[0], self.gQ[1], out=out)
                    out.add_(self.gQ[2])

    def backward_deferred(self, mask):
        lrd, r, st = self.lrd, self.r, self.st
        for l in reversed(range(self.n_layers)):
            L = self.layers[l]
            q, o, up, dn = L["qkv"], L["o"], L["up"], L["dn"]
            lrd.linear_bwd_data(self.G[l], dn["V"], dn["U"], self.gZ[l], dn["dH"], L["Z"], lrd.ACT_GELU, self.ws)
            lrd.linear_bwd_data(self.gZ[l], up["V"], up["U"], self.gXo[l], up["dH"], None, lrd.ACT_NONE, self.ws)
            lrd.linear_bwd_data(self.gXo[l], o["V"], o["U"], self.gAttn, o["dH"], None, lrd.ACT_NONE, self.ws)
            lrd.linear_group_bwd_data(L["dqkv"], q["V"], q["U"], self.G[l - 1] if l > 0 else None, q["dH"], self.ws)
        tu, tv = not mask & 2, not mask & 1
        for name, dY, X in (("dn", self.G, self.A), ("up", self.gZ, self.Xo), ("o", self.gXo, self.attn)):
            s = st[name]
            lrd.linear_wgrad_batched(dY if tu else None, s["H"] if tu else None, s["dH"] if tv else None, X if tv else None,
                                     s["dV"], s["dU"], mask, self.ws)
        q = st["qkv"]
        if tv:      # the stacked first factors: one product of depth 3r per layer
            lrd.linear_wgrad_batched(None, None, q["dH"], self.Xs, q["dV"], None, mask | 2, self.ws)
        if tu:      # the second factors: member g of every layer, addressed inside the stacks
            for g in range(3):
                lrd.linear_wgrad_batched(self.dqkv[:, g], q["H"][:, :, g * r:(g + 1) * r], None, None, None, q["dU_by_member"][g],
                                         mask | 1, self.ws)

    def step(self, mask):
        self.forward()
        self.backward(mask)

    def passes(self, mask):
        """(name, flops, algorithmic bytes) of every layer pass (forward + backward of one call site) of a step."""
        T, d, ff, r = ENC_T, ENC_D, ENC_FF, self.r
        out = []
        for l in range(self.n_layers):
            first = l == 0
            # Q/K/V: three pairs sharing X (read once) and producing one dX (written once)
            f, b = layer_flops(T, d, d, r, mask, want_dx=not first)
            e = 2
            by = e * T * d + 3 * e * (T * d + 2 * r * d)                      # forward: X, three results, three factor pairs
            by += 3 * e * (T * d + 2 * r * d) + (0 if first else e * T * d)   # backward: three gradients in, factors, one dX out
            if not mask & 1:
                by += e * T * d + 3 * 4 * r * d                               # X again and the fp32 gradients of the first factors
            if not mask & 2:
                by += 2 * e * T * 3 * r + 3 * 4 * r * d                       # H saved and re-read, gradients of the second factors
            out.append(("qkv", 3 * (f + b), by))
            for name, n_in, n_out, ao, ai in (("o", d, d, False, False), ("up", d, ff, True, False), ("dn", ff, d, False, True)):
                f, b = layer_flops(T, n_in, n_out, r, mask)
                byf, byb = linear_bytes(T, n_in, n_out, r, mask, act_out=ao, act_in=ai)
                out.append((name, f + b, byf + byb))
        return out

    def flops(self, mask):
        return sum(f for _, f, _ in self.passes(mask))

    def roof_us(self, mask):
        return sum(roof_us(f, b)[0] for _, f, b in self.passes(mask))


class DenseEncoder:
    """The same layers undecomposed (the original network's linears)."""

    def __init__(self, lrd, torch, np, si, layers=ENC_LAYERS):
        self.lrd, self.n_layers = lrd, layers
        dev, bf = "cuda", torch.bfloat16
        rng = si.rng_for(5, 77)
        T, d, ff = ENC_T, ENC_D, ENC_FF

        def to_dev(a):
            bits = si.bf16_bits(a).view(np.int16)
            return torch.from_numpy(bits).to(dev).view(bf).reshape(a.shape)

        def empty(*shape, dt=bf):
            return torch.empty(shape, dtype=dt, device=dev)

        self.layers = [dict(Wqkv=to_dev(si.linear_weight(3 * d, d, rng)), Wo=to_dev(si.linear_weight(d, d, rng)),
                            Wup=to_dev(si.linear_weight(ff, d, rng)), Wdn=to_dev(si.linear_weight(d, ff, rng)),
                            attn=to_dev(si.gaussian((T, d), rng)), dqkv=to_dev(si.gaussian((T, 3 * d), rng, 1e-2)),
                            Yqkv=empty(T, 3 * d), Xo=empty(T, d), Z=empty(T, ff), A=empty(T, ff)) for _ in range(layers)]
        self.dW = dict(qkv=empty(3 * d, d, dt=torch.float32), o=empty(d, d, dt=torch.float32), up=empty(ff, d, dt=torch.float32),
                       dn=empty(d, ff, dt=torch.float32))
        self.X = [to_dev(si.gaussian((T, d), rng))] + [empty(T, d) for _ in range(layers)]
        self.gX = [empty(T, d) for _ in range(2)]
        self.gXo, self.gAttn, self.gA, self.gZ = empty(T, d), empty(T, d), empty(T, ff), empty(T, ff)
        nbytes = max(lrd.dense_linear_workspace_bytes(T, d, 3 * d, lrd.BF16), lrd.dense_linear_workspace_bytes(T, d, ff, lrd.BF16),
                     lrd.dense_linear_workspace_bytes(T, ff, d, lrd.BF16))
        self.ws = torch.empty(nbytes + 256, dtype=torch.uint8, device=dev)

    def step(self, mask=0):
        lrd = self.lrd
        for l, L in enumerate(self.layers):
            lrd.dense_linear_fwd(self.X[l], L["Wqkv"], None, L["Yqkv"], self.ws)
            lrd.dense_linear_fwd(L["attn"], L["Wo"], None, L["Xo"], self.ws)
            lrd.dense_linear_fwd(L["Xo"], L["Wup"], None, L["Z"], self.ws)
            lrd.gelu_fwd(L["Z"], L["A"])
            lrd.dense_linear_fwd(L["A"], L["Wdn"], None, self.X[l + 1], self.ws)
        g = self.X[self.n_layers]
        for l in reversed(range(self.n_layers)):
            L = self.layers[l]
            out = self.gX[l & 1]
            lrd.dense_linear_bwd(g, L["A"], L["Wdn"], self.gA, self.dW["dn"], self.ws)
            lrd.gelu_bwd(self.gA, L["Z"], self.gZ)
            lrd.dense_linear_bwd(self.gZ, L["Xo"], L["Wup"], self.gXo, self.dW["up"], self.ws)
            lrd.dense_linear_bwd(self.gXo, L["attn"], L["Wo"], self.gAttn, self.dW["o"], self.ws)
            lrd.dense_linear_bwd(L["dqkv"], self.X[l], L["Wqkv"], out if l > 0 else None, self.dW["qkv"], self.ws)
            g = out

    def flops(self):
        T, d, ff = ENC_T, ENC_D, ENC_FF
        per = 6 * T * (3 * d * d + d * d + 2 * d * ff)
        return self.n_layers * per - 2 * T * 3 * d * d          # layer 0 has no input gradient


def timed(torch, fn, steps, warmup, first_step=0):
    for s in range(warmup):
        fn(s)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(first_step, first_step + steps):
        fn(s)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def graph_timed(torch, step_for_parity, steps, warmup):
    """ms per step of `steps` replays of captured HIP graphs (one per freeze parity, alternating)."""
    graphs = []
    side = torch.cuda.Stream()
    for parity in (0, 1):
        step_for_parity(parity)                      # eager run first: first-call set-up stays out of the capture
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            step_for_parity(parity)
        graphs.append(g)
    torch.cuda.synchronize()
    return timed(torch, lambda s: graphs[s & 1].replay(), steps, warmup)


def cpu_baseline(np, si, oracle, rank, layers=6):
    """The fp64 oracle, as it stands, on `layers` of the 12 encoder layers at all tokens (forward +
    backward, first factors frozen), the same chain of layer calls as the device step."""
    rng = si.rng_for(5, 99)
    T, d, ff = ENC_T, ENC_D, ENC_FF
    mask = oracle.freeze_mask(oracle.KIND_SVD, 0)
    rb = si.round_bf16

    def pair(n_out, n_in):
        U, V = si.direct_factors(n_out, n_in, rank, rng)
        return rb(U), rb(V)

    net = [dict(qkv=[pair(d, d) for _ in range(3)], o=pair(d, d), up=pair(ff, d), dn=pair(d, ff),
                attn=rb(si.gaussian((T, d), rng)), dqkv=rb(si.gaussian((3, T, d), rng, 1e-2))) for _ in range(layers)]
    x = rb(si.gaussian((T, d), rng))
    t0 = time.perf_counter()
    saved = []
    for L in net:
        hq = [oracle.linear_fwd(x, V, U)[0] for U, V in L["qkv"]]
        ho, xo = oracle.linear_fwd(L["attn"], L["o"][1], L["o"][0])
        hu, z = oracle.linear_fwd(xo, L["up"][1], L["up"][0])
        a = oracle.gelu_fwd(z)
        hd, y = oracle.linear_fwd(a, L["dn"][1], L["dn"][0])
        saved.append((x, hq, ho, xo, hu, z, a, hd))
        x = y
    g = x
    for l in reversed(range(layers)):
        L = net[l]
        x0, hq, ho, xo, hu, z, a, hd = saved[l]
        gz = oracle.gelu_bwd(oracle.linear_bwd(g, a, hd, L["dn"][1], L["dn"][0], mask)["dX"], z)
        gxo = oracle.linear_bwd(gz, xo, hu, L["up"][1], L["up"][0], mask)["dX"]
        oracle.linear_bwd(gxo, L["attn"], ho, L["o"][1], L["o"][0], mask)
        gx = 0.0
        for (U, V), h, dy in zip(L["qkv"], hq, L["dqkv"]):
            gx = gx + oracle.linear_bwd(dy, x0, h, V, U, mask)["dX"]
        g = gx
    dt = time.perf_counter() - t0
    flops = 0
    for _ in range(layers):
        for n_in, n_out, n in ((d, d, 4), (d, ff, 1), (ff, d, 1)):
            f, b = layer_flops(T, n_in, n_out, rank, mask)
            flops += n * (f + b)
    return dict(value=flops / dt / 1e12, unit="TFLOP/s", cores=oracle.threads(), kind="oracle",
                sample=f"{layers} of {ENC_LAYERS} encoder layers, all {T} tokens, fwd+bwd with first factors frozen, fp64; {dt:.1f} s",
                tokens_per_s=T / (dt * ENC_LAYERS / layers))


def rank_sweep(args, torch, lrd):
    """Config 3: one 4096 x 4096 linear, 16384 tokens, bf16; forward + backward time against the rank
    (raw ranks and their quantized neighbours) with nothing / V / U frozen, beside the dense layer.
    Timing only (tests/test_gpu_fullsize.py compares this layer with the oracle at r = 257, 512, 513, 768, 1024 and
    undecomposed, tests/test_gpu_linear.py at r = 256); prints one JSON line."""
    T, d = 16384, 4096
    bf = torch.bfloat16
    gen = torch.Generator(device="cuda").manual_seed(230903824 + 3)

    def rnd(*shape, scale=1.0):
        return (torch.randn(*shape, device="cuda", generator=gen) * scale).to(bf)

    def timeit(fn, iters):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s.record()
        for _ in range(iters):
            fn()
        e.record()
        torch.cuda.synchronize()
        return s.elapsed_time(e) * 1e3 / iters

    X, dY = rnd(T, d), rnd(T, d)
    Y, dX = torch.empty(T, d, dtype=bf, device="cuda"), torch.empty(T, d, dtype=bf, device="cuda")
    ranks = sorted(set(list(range(args.sweep_step, 1025, args.sweep_step)) +
                       [q + o for q in range(64, 1025, 64) for o in (-1, 0, 1) if 1 <= q + o <= 1024] + [1]))
    ws = torch.empty(max(lrd.linear_workspace_bytes(T, d, d, r, lrd.BF16, 0) for r in ranks) + 256,
                     dtype=torch.uint8, device="cuda")
    points = []
    for r in ranks:
        V, U = rnd(r, d, scale=d ** -0.5), rnd(d, r, scale=r ** -0.5)
        H = torch.empty(T, r, dtype=bf, device="cuda")
        dV, dU = torch.empty(r, d, device="cuda"), torch.empty(d, r, device="cuda")
        fwd = timeit(lambda: lrd.linear_fwd(X, V, U, None, Y, H, ws), args.sweep_iters)
        row = dict(r=r, fwd_us=fwd)
        for name, mask in (("none", 0), ("V", 1), ("U", 2)):
            row[f"bwd_us_frozen_{name}"] = timeit(
                lambda: lrd.linear_bwd(dY, X, H, V, U, dX, dV, dU, None, mask, ws), args.sweep_iters)
        row["tflops_fwd_bwd_V_frozen"] = 10.0 * T * d * r / ((fwd + row["bwd_us_frozen_V"]) * 1e-6) / 1e12
        points.append(row)
    W, dW = rnd(d, d, scale=d ** -0.5), torch.empty(d, d, device="cuda")
    wsd = torch.empty(lrd.dense_linear_workspace_bytes(T, d, d, lrd.BF16) + 256, dtype=torch.uint8, device="cuda")
    dense_f = timeit(lambda: lrd.dense_linear_fwd(X, W, None, Y, wsd), 5)
    dense_b = timeit(lambda: lrd.dense_linear_bwd(dY, X, W, dX, dW, wsd), 5)
    print(json.dumps(dict(metric="rank sweep: decomposed 4096x4096 linear, 16384 tokens, bf16 (fwd / bwd microseconds)",
                          dense=dict(fwd_us=dense_f, bwd_us=dense_b, tflops=6.0 * T * d * d / ((dense_f + dense_b) * 1e-6) / 1e12),
                          points=points)))


def train_step(args, torch, np, si, lrd, factorize):
    """The FFN stack of the headline with the optimizer in the step: forward, then backward with the SGD
    update (momentum 0.9, weight decay 1e-4; Section 3) of every factor the freeze mask leaves
    trainable, through lrd_linear_bwd_sgd.  Replayed from captured graphs like the headline; beside
    it the same step with nothing frozen, and forward + backward without any update.  Prints one JSON line."""
    rank = lrd.quantize_rank(int(0.25 * min(D_MODEL, D_FF)), 64)
    stack = Stack(lrd, torch, np, si, factorize, rank, seed_stream=0, true_svd=False)
    opt = lrd.Sgd(1e-6, 0.9, 1e-4)
    for blk in stack.layers:
        for l in blk:
            l["Um"], l["Vm"] = l["U"].float(), l["V"].float()
            l["mU"], l["mV"] = torch.zeros_like(l["Um"]), torch.zeros_like(l["Vm"])
    nbytes = max(lrd.linear_sgd_workspace_bytes(T_TOKENS, D_MODEL, D_FF, rank, lrd.BF16, 0),
                 lrd.linear_sgd_workspace_bytes(T_TOKENS, D_FF, D_MODEL, rank, lrd.BF16, 0))
    ws = torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda")

    def backward_sgd(mask):
        g = stack.X[N_BLOCKS]
        for b in reversed(range(N_BLOCKS)):
            l1, l2 = stack.layers[b]
            out = stack.gX[b & 1]
            lrd.linear_bwd_sgd(g, stack.A[b], l2["H"], l2["V"], l2["U"], stack.gZ, l2["Vm"], l2["Um"], l2["mV"], l2["mU"], None,
                               mask, stack.Z[b], lrd.ACT_GELU, opt, ws)
            lrd.linear_bwd_sgd(stack.gZ, stack.X[b], l1["H"], l1["V"], l1["U"], out if b > 0 else None, l1["Vm"], l1["Um"],
                               l1["mV"], l1["mU"], None, mask, None, lrd.ACT_NONE, opt, ws)
            g = out

    def with_sgd(masks):
        def run(parity):
            stack.forward()
            backward_sgd(masks[parity])
        return run

    alternating = (lrd.freeze_mask(lrd.KIND_SVD, 0), lrd.freeze_mask(lrd.KIND_SVD, 1))
    res = dict(metric="FFN stack training step with the SGD update in the backward (ms per step, hip-graph replay)",
               rank=rank, tokens=T_TOKENS, blocks=N_BLOCKS)
    res["sequential_freezing_with_sgd_ms"] = graph_timed(torch, with_sgd(alternating), args.steps, args.warmup)
    res["nothing_frozen_with_sgd_ms"] = graph_timed(torch, with_sgd((0, 0)), args.steps, args.warmup)
    res["sequential_freezing_no_update_ms"] = graph_timed(torch, lambda parity: stack.step(alternating[parity]), args.steps, args.warmup)
    res["nothing_frozen_no_update_ms"] = graph_timed(torch, lambda parity: stack.step(0), args.steps, args.warmup)
    res["speedup_freezing_with_sgd"] = res["nothing_frozen_with_sgd_ms"] / res["sequential_freezing_with_sgd_ms"]
    res["speedup_freezing_no_update"] = res["nothing_frozen_no_update_ms"] / res["sequential_freezing_no_update_ms"]
    print(json.dumps(res), flush=True)


def conv_stage(args, torch, lrd):
    """One 3x3 stage of config 4 (N = 128, Tucker ranks C/2) and the dense layer beside it: forward and
    the backward with nothing frozen, a few times, for a kernel trace.  Prints one JSON line."""
    bf = torch.bfloat16
    gen = torch.Generator(device="cuda").manual_seed(230903824 + 4)
    C = args.conv_stage
    hw = {64: 56, 128: 28, 256: 14, 512: 7}[C]
    N, k, r = 128, 3, C // 2

    def rnd(*shape, scale=1.0):
        return (torch.randn(*shape, device="cuda", generator=gen) * scale).to(bf)

    def empty(*shape, dt=bf):
        return torch.empty(*shape, dtype=dt, device="cuda")

    g = lrd.conv_geom(N, hw, hw, C, C, r, r, k, 1, 1)
    X, dY, Y, dX = rnd(N, hw, hw, C), rnd(N, hw, hw, C), empty(N, hw, hw, C), empty(N, hw, hw, C)
    P1, G, P2 = rnd(r, C, scale=C ** -0.5), rnd(r, k, k, r, scale=(k * k * r) ** -0.5), rnd(C, r, scale=r ** -0.5)
    A, B = empty(N, hw, hw, r), empty(N, hw, hw, r)
    dP1, dG, dP2 = empty(r, C, dt=torch.float32), empty(r, k, k, r, dt=torch.float32), empty(C, r, dt=torch.float32)
    W, dW = rnd(C, k, k, C, scale=(k * k * C) ** -0.5), empty(C, k, k, C, dt=torch.float32)
    ws = torch.empty(lrd.tucker_conv_workspace_bytes(g, lrd.BF16, 0) + 256, dtype=torch.uint8, device="cuda")
    wsd = torch.empty(lrd.dense_conv_workspace_bytes(g, lrd.BF16) + 256, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    iters = 5
    for _ in range(iters):
        lrd.tucker_conv_fwd(X, P1, G, P2, Y, A, B, g, ws)
        lrd.tucker_conv_bwd(dY, X, A, B, P1, G, P2, dX, dP1, dG, dP2, 0, g, ws)
    for _ in range(iters):
        lrd.dense_conv_fwd(X, W, Y, g, wsd)
        lrd.dense_conv_bwd(dY, X, W, dX, dW, g, wsd)
    torch.cuda.synchronize()
    print(json.dumps(dict(metric="conv stage kernel trace run", C=C, hw=hw, N=N, r=r, iters=iters)), flush=True)


def layer_tables(args, torch, lrd):
    """Configs 4 and 5, layer by layer: the four ResNet-style 3x3 stages (N = 128, Tucker ranks C/2 and
    the raw ranks next to them, core frozen / 1x1s frozen / nothing frozen, beside the dense conv) and
    the transformer projections 1024->1024, 1024->4096, 4096->1024 (8192 tokens, r = 256).
    Timing only (parity of these shapes is covered by the tests); prints one JSON line."""
    bf = torch.bfloat16
    gen = torch.Generator(device="cuda").manual_seed(230903824 + 4)

    def rnd(*shape, scale=1.0):
        return (torch.randn(*shape, device="cuda", generator=gen) * scale).to(bf)

    def timeit(fn, iters=10):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s.record()
        for _ in range(iters):
            fn()
        e.record()
        torch.cuda.synchronize()
        return s.elapsed_time(e) * 1e3 / iters

    def empty(*shape, dt=bf):
        return torch.empty(*shape, dtype=dt, device="cuda")

    conv = []
    N, k = 128, 3
    for C, hw in ((64, 56), (128, 28), (256, 14), (512, 7)):
        X, dY = rnd(N, hw, hw, C), rnd(N, hw, hw, C)
        Y, dX = empty(N, hw, hw, C), empty(N, hw, hw, C)
        P = N * hw * hw
        stage = dict(C=C, hw=hw, pixels=P, ranks=[])
        for r in (C // 2 - 1, C // 2, C // 2 + 1):
            g = lrd.conv_geom(N, hw, hw, C, C, r, r, k, 1, 1)
            P1, G, P2 = rnd(r, C, scale=C ** -0.5), rnd(r, k, k, r, scale=(k * k * r) ** -0.5), rnd(C, r, scale=r ** -0.5)
            A, B = empty(N, hw, hw, r), empty(N, hw, hw, r)
            dP1, dG, dP2 = empty(r, C, dt=torch.float32), empty(r, k, k, r, dt=torch.float32), empty(C, r, dt=torch.float32)
            ws = torch.empty(lrd.tucker_conv_workspace_bytes(g, lrd.BF16, 0) + 256, dtype=torch.uint8, device="cuda")
            fwd = timeit(lambda: lrd.tucker_conv_fwd(X, P1, G, P2, Y, A, B, g, ws))
            row = dict(r=r, fwd_us=fwd)
            for name, mask in (("core", 0b010), ("1x1", 0b101), ("none", 0)):
                row[f"bwd_us_frozen_{name}"] = timeit(
                    lambda: lrd.tucker_conv_bwd(dY, X, A, B, P1, G, P2, dX, dP1, dG, dP2, mask, g, ws))
            f_fwd = 2.0 * P * (C * r + k * k * r * r + r * C)
            f_bwd_core = 2.0 * f_fwd - 2.0 * P * k * k * r * r
            row["tflops_fwd_bwd_core_frozen"] = (f_fwd + f_bwd_core) / ((fwd + row["bwd_us_frozen_core"]) * 1e-6) / 1e12
            # algorithmic bytes, core frozen: X, Y, dY, dX once each; A, B written and read back; factors; fp32 1x1 gradients
            byts = 2.0 * (4 * P * C + 4 * P * r) + 2.0 * (2 * C * r + k * k * r * r) + 4.0 * 2 * C * r
            row["hbm_frac_fwd_bwd_core_frozen"] = byts / ((fwd + row["bwd_us_frozen_core"]) * 1e-6) / 1e9 / HBM_PEAK_GBS
            stage["ranks"].append(row)
        g = lrd.conv_geom(N, hw, hw, C, C, C // 2, C // 2, k, 1, 1)
        W, dW = rnd(C, k, k, C, scale=(k * k * C) ** -0.5), empty(C, k, k, C, dt=torch.float32)
        wsd = torch.empty(lrd.dense_conv_workspace_bytes(g, lrd.BF16) + 256, dtype=torch.uint8, device="cuda")
        stage["dense_fwd_us"] = timeit(lambda: lrd.dense_conv_fwd(X, W, Y, g, wsd), 5)
        stage["dense_bwd_us"] = timeit(lambda: lrd.dense_conv_bwd(dY, X, W, dX, dW, g, wsd), 5)
        stage["dense_tflops"] = 6.0 * P * k * k * C * C / ((stage["dense_fwd_us"] + stage["dense_bwd_us"]) * 1e-6) / 1e12
        conv.append(stage)

    # stride-2 3x3 layers between the stages (C -> 2C, ranks C/2 and C), aligned ranks only
    trans = []
    for C, hw in ((64, 56), (128, 28), (256, 14)):
        S, r1, r2, ho = 2 * C, C // 2, C, hw // 2
        g = lrd.conv_geom(N, hw, hw, C, S, r1, r2, k, 2, 1)
        X, dY = rnd(N, hw, hw, C), rnd(N, ho, ho, S)
        Y, dX = empty(N, ho, ho, S), empty(N, hw, hw, C)
        P1, G, P2 = rnd(r1, C, scale=C ** -0.5), rnd(r2, k, k, r1, scale=(k * k * r1) ** -0.5), rnd(S, r2, scale=r2 ** -0.5)
        A, B = empty(N, hw, hw, r1), empty(N, ho, ho, r2)
        dP1, dG, dP2 = empty(r1, C, dt=torch.float32), empty(r2, k, k, r1, dt=torch.float32), empty(S, r2, dt=torch.float32)
        ws = torch.empty(lrd.tucker_conv_workspace_bytes(g, lrd.BF16, 0) + 256, dtype=torch.uint8, device="cuda")
        row = dict(C=C, S=S, hw=hw, r1=r1, r2=r2, fwd_us=timeit(lambda: lrd.tucker_conv_fwd(X, P1, G, P2, Y, A, B, g, ws)))
        for name, mask in (("core", 0b010), ("1x1", 0b101), ("none", 0)):
            row[f"bwd_us_frozen_{name}"] = timeit(
                lambda: lrd.tucker_conv_bwd(dY, X, A, B, P1, G, P2, dX, dP1, dG, dP2, mask, g, ws))
        W, dW = rnd(S, k, k, C, scale=(k * k * C) ** -0.5), empty(S, k, k, C, dt=torch.float32)
        wsd = torch.empty(lrd.dense_conv_workspace_bytes(g, lrd.BF16) + 256, dtype=torch.uint8, device="cuda")
        row["dense_fwd_us"] = timeit(lambda: lrd.dense_conv_fwd(X, W, Y, g, wsd), 5)
        row["dense_bwd_us"] = timeit(lambda: lrd.dense_conv_bwd(dY, X, W, dX, dW, g, wsd), 5)
        trans.append(row)

    lin = []
    T, r = 8192, 256
    for n_in, n_out in ((1024, 1024), (1024, 4096), (4096, 1024)):
        X, dY = rnd(T, n_in), rnd(T, n_out)
        V, U = rnd(r, n_in, scale=n_in ** -0.5), rnd(n_out, r, scale=r ** -0.5)
        Y, H, dX = empty(T, n_out), empty(T, r), empty(T, n_in)
        dV, dU = empty(r, n_in, dt=torch.float32), empty(n_out, r, dt=torch.float32)
        ws = torch.empty(lrd.linear_workspace_bytes(T, n_in, n_out, r, lrd.BF16, 0) + 256, dtype=torch.uint8, device="cuda")
        fwd = timeit(lambda: lrd.linear_fwd(X, V, U, None, Y, H, ws), 20)
        row = {"in": n_in, "out": n_out, "r": r, "fwd_us": fwd}
        for name, mask in (("V", 1), ("U", 2), ("none", 0)):
            row[f"bwd_us_frozen_{name}"] = timeit(lambda: lrd.linear_bwd(dY, X, H, V, U, dX, dV, dU, None, mask, ws), 20)
        f_v = 2.0 * T * r * (n_in + n_out) * 2 + 2.0 * T * r * n_out
        row["tflops_fwd_bwd_V_frozen"] = f_v / ((fwd + row["bwd_us_frozen_V"]) * 1e-6) / 1e12
        W, dW = rnd(n_out, n_in, scale=n_in ** -0.5), empty(n_out, n_in, dt=torch.float32)
        wsd = torch.empty(lrd.dense_linear_workspace_bytes(T, n_in, n_out, lrd.BF16) + 256, dtype=torch.uint8, device="cuda")
        row["dense_fwd_us"] = timeit(lambda: lrd.dense_linear_fwd(X, W, None, Y, wsd), 10)
        row["dense_bwd_us"] = timeit(lambda: lrd.dense_linear_bwd(dY, X, W, dX, dW, wsd), 10)
        lin.append(row)
    # query / key / value projections of one attention block: three separate layers (their data gradients
    # added afterwards) against the grouped call with the stacked first factor
    G3, n_in, n_out = 3, 1024, 1024
    X = rnd(T, n_in)
    dY3 = rnd(G3, T, n_out)
    V_cat, U3 = rnd(G3 * r, n_in, scale=n_in ** -0.5), rnd(G3, n_out, r, scale=r ** -0.5)
    Y3, H3 = empty(G3, T, n_out), empty(T, G3 * r)
    Hs = [empty(T, r) for _ in range(G3)]
    dX, dXg = empty(T, n_in), [empty(T, n_in) for _ in range(G3)]
    dV3, dU3 = empty(G3 * r, n_in, dt=torch.float32), empty(G3, n_out, r, dt=torch.float32)
    ws = torch.empty(max(lrd.linear_group_workspace_bytes(T, n_in, n_out, r, G3, lrd.BF16, 0),
                         lrd.linear_workspace_bytes(T, n_in, n_out, r, lrd.BF16, 0)) + 256, dtype=torch.uint8, device="cuda")

    def separate(mask):
        for g in range(G3):
            lrd.linear_fwd(X, V_cat[g * r:(g + 1) * r], U3[g], None, Y3[g], Hs[g], ws)
        for g in range(G3):
            lrd.linear_bwd(dY3[g], X, Hs[g], V_cat[g * r:(g + 1) * r], U3[g], dXg[g], dV3[g * r:(g + 1) * r], dU3[g], None,
                           mask, ws)
        torch.add(dXg[0], dXg[1], out=dX)
        dX.add_(dXg[2])

    def grouped(mask):
        lrd.linear_group_fwd(X, V_cat, U3, None, Y3, H3, ws)
        lrd.linear_group_bwd(dY3, X, H3, V_cat, U3, dX, dV3, dU3, None, mask, ws)

    qkv = dict(T=T, r=r, groups=G3, **{"in": n_in, "out": n_out})
    for name, mask in (("V", 1), ("U", 2), ("none", 0)):
        qkv[f"separate_us_frozen_{name}"] = timeit(lambda: separate(mask), 20)
        qkv[f"grouped_us_frozen_{name}"] = timeit(lambda: grouped(mask), 20)

    print(json.dumps(dict(metric="layer tables: config 4 (Tucker 3x3 stages, N = 128) and config 5 (projections, 8192 tokens, r = 256), "
                                 "bf16, microseconds per call", conv_stages=conv, stride2_transitions=trans, projections=lin, qkv=qkv)))


def rank_search(args, torch, lrd):
    """Algorithm 1 (rank optimization) run on the device: step time (forward + backward, nothing frozen)
    of every rank from the estimated one (eq. 6 at compression alpha = 2) down to the lower bound (eq. 7,
    alpha + 1), lrd_select_rank on the measured curve, and the aligned ranks lrd_quantize_rank would have
    picked, for the paper's [512,512,3,3] Tucker layer (N = 128, 7 x 7) and the 4096 x 4096 linear layer
    (16384 tokens).  Timing only; prints one JSON line."""
    bf = torch.bfloat16
    gen = torch.Generator(device="cuda").manual_seed(230903824 + 6)

    def rnd(*shape, scale=1.0):
        return (torch.randn(*shape, device="cuda", generator=gen) * scale).to(bf)

    def empty(*shape, dt=bf):
        return torch.empty(*shape, dtype=dt, device="cuda")

    def timeit(fn, iters):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s.record()
        for _ in range(iters):
            fn()
        e.record()
        torch.cuda.synchronize()
        return s.elapsed_time(e) * 1e3 / iters

    def report(name, ranks, times, t_dense, extra):
        r_min, r_max = ranks[0], ranks[-1]
        noise = 0.03 * sorted(times)[len(times) // 2]      # differences below 3 % of the median step are jitter
        out = dict(layer=name, r_estimated=r_max, r_min=r_min, dense_us=t_dense, noise_us=noise,
                   t_estimated_us=times[-1], **extra)
        for label, mode in (("first_peak", lrd.SELECT_FIRST_PEAK), ("argmax", lrd.SELECT_ARGMAX),
                            ("first_peak_require_faster", lrd.SELECT_FIRST_PEAK | lrd.SELECT_REQUIRE_FASTER)):
            r_opt, keep = lrd.select_rank(times, r_min, r_max, t_dense, noise, mode)
            out[label] = dict(r_opt=r_opt, keep_decomposed=keep, t_us=times[r_opt - r_min],
                              speedup_vs_estimated=times[-1] / times[r_opt - r_min],
                              speedup_vs_dense=t_dense / times[r_opt - r_min])
        out["quantize_down"] = {str(m): dict(r=lrd.quantize_rank(r_max, m, lrd.ROUND_DOWN, r_min, r_max),
                                             t_us=times[lrd.quantize_rank(r_max, m, lrd.ROUND_DOWN, r_min, r_max) - r_min])
                                for m in (8, 16, 32, 64)}
        out["curve_us"] = [round(t, 1) for t in times]
        return out

    results = []
    # --- the paper's worked example: [512,512,3,3], Tucker-2 at 2x compression
    C, k, N, hw = 512, 3, 128, 7
    R, _ = lrd.tucker_rank(C, C, k, 2.0, 1.0)
    R_min, _ = lrd.tucker_rank(C, C, k, 3.0, 1.0)
    X, dY = rnd(N, hw, hw, C), rnd(N, hw, hw, C)
    Y, dX = empty(N, hw, hw, C), empty(N, hw, hw, C)
    ranks = list(range(R_min, R + 1))
    gmax = lrd.conv_geom(N, hw, hw, C, C, R, R, k, 1, 1)
    ws = torch.empty(max(lrd.tucker_conv_workspace_bytes(lrd.conv_geom(N, hw, hw, C, C, r, r, k, 1, 1), lrd.BF16, 0)
                         for r in ranks) + 256, dtype=torch.uint8, device="cuda")
    times = []
    for r in ranks:
        g = lrd.conv_geom(N, hw, hw, C, C, r, r, k, 1, 1)
        P1, G, P2 = rnd(r, C, scale=C ** -0.5), rnd(r, k, k, r, scale=(k * k * r) ** -0.5), rnd(C, r, scale=r ** -0.5)
        A, B = empty(N, hw, hw, r), empty(N, hw, hw, r)
        dP1, dG, dP2 = empty(r, C, dt=torch.float32), empty(r, k, k, r, dt=torch.float32), empty(C, r, dt=torch.float32)

        def step():
            lrd.tucker_conv_fwd(X, P1, G, P2, Y, A, B, g, ws)
            lrd.tucker_conv_bwd(dY, X, A, B, P1, G, P2, dX, dP1, dG, dP2, 0, g, ws)
        times.append(timeit(step, args.sweep_iters))
    W, dW = rnd(C, k, k, C, scale=(k * k * C) ** -0.5), empty(C, k, k, C, dt=torch.float32)
    wsd = torch.empty(lrd.dense_conv_workspace_bytes(gmax, lrd.BF16) + 256, dtype=torch.uint8, device="cuda")

    def dense_step():
        lrd.dense_conv_fwd(X, W, Y, gmax, wsd)
        lrd.dense_conv_bwd(dY, X, W, dX, dW, gmax, wsd)
    results.append(report("tucker [512,512,3,3], N=128, 7x7", ranks, times, timeit(dense_step, args.sweep_iters),
                          dict(alpha=2.0)))
    del X, dY, Y, dX, ws, wsd

    # --- the 4096 x 4096 linear layer at 2x compression
    T, d = 16384, 4096
    R, R_min = lrd.svd_rank(d, d, 2.0), lrd.svd_rank(d, d, 3.0)
    X, dY = rnd(T, d), rnd(T, d)
    Y, dX = empty(T, d), empty(T, d)
    ranks = list(range(R_min, R + 1))
    ws = torch.empty(max(lrd.linear_workspace_bytes(T, d, d, r, lrd.BF16, 0) for r in (R, R - 1)) + 256,
                     dtype=torch.uint8, device="cuda")
    times = []
    for r in ranks:
        V, U = rnd(r, d, scale=d ** -0.5), rnd(d, r, scale=r ** -0.5)
        H = empty(T, r)
        dV, dU = empty(r, d, dt=torch.float32), empty(d, r, dt=torch.float32)

        def step():
            lrd.linear_fwd(X, V, U, None, Y, H, ws)
            lrd.linear_bwd(dY, X, H, V, U, dX, dV, dU, None, 0, ws)
        times.append(timeit(step, max(2, args.sweep_iters // 2)))
    W, dW = rnd(d, d, scale=d ** -0.5), empty(d, d, dt=torch.float32)
    wsd = torch.empty(lrd.dense_linear_workspace_bytes(T, d, d, lrd.BF16) + 256, dtype=torch.uint8, device="cuda")

    def dense_lin():
        lrd.dense_linear_fwd(X, W, None, Y, wsd)
        lrd.dense_linear_bwd(dY, X, W, dX, dW, wsd)
    results.append(report("linear 4096x4096, 16384 tokens", ranks, times, timeit(dense_lin, 5), dict(alpha=2.0)))
    print(json.dumps(dict(metric="rank search (Algorithm 1) on measured forward + backward step times, bf16, microseconds",
                          layers=results)))


def factorize_bench(args, torch, np, si, lrd):
    """The one-time factorization on the device (lrd_svd_factors, lrd_tucker2_factors) on the workload's
    layer shapes, beside LAPACK on the host cores for the same matrices; prints one JSON line."""
    import time as _t
    rows = []

    def clock(fn):
        torch.cuda.synchronize()
        t0 = _t.perf_counter()
        out = fn()
        torch.cuda.synchronize()
        return (_t.perf_counter() - t0) * 1e3, out

    for n_out, n_in, r in ((3072, 768, 192), (768, 3072, 192), (1024, 1024, 256), (4096, 4096, 1024)):
        rng = si.rng_for(6, n_out + n_in)
        W = si.linear_weight(n_out, n_in, rng).astype(np.float32)
        Wd = torch.from_numpy(W).cuda()
        U = torch.empty((n_out, r), dtype=torch.float32, device="cuda")
        V = torch.empty((r, n_in), dtype=torch.float32, device="cuda")
        ws = torch.empty(lrd.svd_factors_workspace_bytes(n_out, n_in) + 256, dtype=torch.uint8, device="cuda")
        ms, (sig, sweeps) = clock(lambda: lrd.svd_factors(Wd, r, U, V, ws))
        t0 = _t.perf_counter()
        s_host = np.linalg.svd(W.astype(np.float64), compute_uv=True, full_matrices=False)[1]
        host_ms = (_t.perf_counter() - t0) * 1e3
        err = float(torch.linalg.norm(Wd.double() - U.double() @ V.double()) / torch.linalg.norm(Wd.double()))
        best = float(np.sqrt(np.sum(s_host[r:] ** 2) / np.sum(s_host ** 2)))
        rows.append(dict(kind="svd", out=n_out, **{"in": n_in}, r=r, gpu_ms=ms, sweeps=sweeps, host_lapack_fp64_ms=host_ms,
                         rel_error=err, eckart_young_bound=best,
                         sigma_max_rel_diff=float(np.max(np.abs(np.array(sig) - s_host)) / s_host[0])))
    for S, C, k, r1 in ((64, 64, 3, 32), (256, 256, 3, 128), (512, 512, 3, 256)):
        rng = si.rng_for(6, S + C + k)
        W = si.conv_weight(S, C, k, rng).astype(np.float32)
        Wd = torch.from_numpy(W).cuda()
        P1 = torch.empty((r1, C), dtype=torch.float32, device="cuda")
        G = torch.empty((r1, k, k, r1), dtype=torch.float32, device="cuda")
        P2 = torch.empty((S, r1), dtype=torch.float32, device="cuda")
        ws = torch.empty(lrd.tucker2_factors_workspace_bytes(S, C, k) + 256, dtype=torch.uint8, device="cuda")
        ms, sweeps = clock(lambda: lrd.tucker2_factors(Wd, r1, r1, P1, G, P2, ws))
        t0 = _t.perf_counter()
        W64 = W.astype(np.float64)
        np.linalg.svd(W64.transpose(3, 0, 1, 2).reshape(C, -1), full_matrices=False)
        np.linalg.svd(W64.reshape(S, -1), full_matrices=False)
        host_ms = (_t.perf_counter() - t0) * 1e3
        rec = torch.einsum("ob,buva,ac->ouvc", P2.double(), G.double(), P1.double())
        err = float(torch.linalg.norm(Wd.double() - rec) / torch.linalg.norm(Wd.double()))
        rows.append(dict(kind="tucker2", S=S, C=C, k=k, r1=r1, r2=r1, gpu_ms=ms, sweeps=sweeps,
                         host_lapack_fp64_ms=host_ms, rel_error=err))
    # the 24 weights of the FFN stack (12 x 3072x768 and 12 x 768x3072) as two batched calls, against 24 single calls
    for n_out, n_in, r in ((3072, 768, 192), (768, 3072, 192)):
        B = 12
        rng = si.rng_for(6, 9000 + n_out)
        Wb = torch.from_numpy(np.stack([si.linear_weight(n_out, n_in, rng).astype(np.float32) for _ in range(B)])).cuda()
        U = torch.empty((B, n_out, r), dtype=torch.float32, device="cuda")
        V = torch.empty((B, r, n_in), dtype=torch.float32, device="cuda")
        wsb = torch.empty(lrd.svd_factors_batched_workspace_bytes(B, n_out, n_in) + 256, dtype=torch.uint8, device="cuda")
        ms_b, (_, sweeps) = clock(lambda: lrd.svd_factors_batched(Wb, r, U, V, wsb))
        ws1 = torch.empty(lrd.svd_factors_workspace_bytes(n_out, n_in) + 256, dtype=torch.uint8, device="cuda")
        ms_1, _ = clock(lambda: [lrd.svd_factors(Wb[b], r, U[b], V[b], ws1) for b in range(B)])
        rows.append(dict(kind="svd batch of 12", out=n_out, **{"in": n_in}, r=r, batched_ms=ms_b, twelve_single_calls_ms=ms_1, sweeps=sweeps))
    print(json.dumps(dict(metric="one-time factorization on the device (fp64 one-sided Jacobi), milliseconds", cases=rows)))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=4)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-comparators", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="time eager launches only")
    ap.add_argument("--no-workloads", action="store_true", help="skip the other workloads (FFN stack, rank sweep points, Tucker stages)")
    ap.add_argument("--per-layer-backward", action="store_true",
                    help="headline with one backward call per layer instead of batched weight gradients")
    ap.add_argument("--no-peaks", action="store_true", help="skip the in-run peak measurements")
    ap.add_argument("--rank-sweep", action="store_true", help="run the rank sweep (config 3) instead of the FFN stack")
    ap.add_argument("--rank-search", action="store_true",
                    help="run Algorithm 1's rank search on measured step times (Tucker [512,512,3,3] and linear 4096^2) instead")
    ap.add_argument("--factorize", action="store_true", help="time the on-device factorization (SVD pairs, Tucker-2) instead")
    ap.add_argument("--layer-tables", action="store_true",
                    help="time the Tucker conv stages (config 4) and the transformer projections (config 5) instead")
    ap.add_argument("--train-step", action="store_true",
                    help="time the FFN stack with the SGD update inside the backward (lrd_linear_bwd_sgd) instead")
    ap.add_argument("--conv-stage", type=int, default=0, choices=(0, 64, 128, 256, 512),
                    help="run one 3x3 stage of config 4 (Tucker and dense, forward + backward) a few times, for a kernel trace")
    ap.add_argument("--sweep-step", type=int, default=16)
    ap.add_argument("--sweep-iters", type=int, default=5)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three plain 256 MiB device copies (reference for rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import synth_inputs as si
    from paper_2309_03824_amd import binding as lrd
    from paper_2309_03824_amd import factorize

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)

    if args.rank_sweep:
        rank_sweep(args, torch, lrd)
        return
    if args.train_step:
        train_step(args, torch, np, si, lrd, factorize)
        return
    if args.conv_stage:
        conv_stage(args, torch, lrd)
        return
    if args.layer_tables:
        layer_tables(args, torch, lrd)
        return
    if args.rank_search:
        rank_search(args, torch, lrd)
        return
    if args.factorize:
        factorize_bench(args, torch, np, si, lrd)
        return

    if args.calibrate_copy:
        src = torch.ones(1 << 27, dtype=torch.bfloat16, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    out = headline(args, torch, np, si, lrd)
    print(json.dumps(out))


def event_us(torch, fn, iters, warm=2):
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    s.record()
    for _ in range(iters):
        fn()
    e.record()
    torch.cuda.synchronize()
    return s.elapsed_time(e) * 1e3 / iters


def measure_peaks(torch, lrd):
    """What this machine delivers, in this run, to a register-only loop of bf16 matrix instructions and
    to a plain 16-byte-per-lane streaming kernel over 1 GiB (cold: far beyond every cache)."""
    sink = torch.empty(4096 * 256, dtype=torch.float32, device="cuda")
    res = {}
    for wgs in (1024, 4096):
        fl = [0.0]

        def run():
            fl[0] = lrd.measure_mfma_loop(sink, wgs, 2048)
        us = event_us(torch, run, 3)
        res[f"mfma_bf16_loop_tflops_{wgs}_workgroups"] = fl[0] / (us * 1e-6) / 1e12
    # LDS fragment reads: two workgroups per compute unit on all 256 units
    isink = sink.view(torch.int32)
    lb = [0.0]

    def run_lds():
        lb[0] = lrd.measure_lds_read(isink, 512, 4000)
    us = event_us(torch, run_lds, 3)
    res["lds_read_16B_fragments_bytes_per_ns_per_cu"] = lb[0] / 256 / (us * 1e3)
    n = 1 << 30
    a = torch.empty(n, dtype=torch.uint8, device="cuda")
    b = torch.empty(n, dtype=torch.uint8, device="cuda")
    a.zero_()
    for name, mode, moved in (("read", lrd.STREAM_READ, n), ("write", lrd.STREAM_WRITE, n), ("copy", lrd.STREAM_COPY, 2 * n)):
        us = event_us(torch, lambda: lrd.measure_stream(a, b, n, mode), 5)
        res[f"stream_{name}_gbs"] = moved / (us * 1e-6) / 1e9
    res["note"] = ("measured in this run with the library's own measurement kernels (lrd_measure.h); published peaks used for "
                   "the roofline fractions: 2500 TFLOP/s bf16 MFMA, 8000 GB/s HBM")
    return res


# HBM bytes per launch of the product kernels as the traffic counters saw them (FETCH_SIZE, WRITE_SIZE per
# dispatch, scaled by what the same counters read for a plain copy of known size: 2.00 and 1.00), by kernel
# and product shape; profiles/encoder_step_hbm_traffic.md holds the runs.  Reported only for a kernel and a
# mix of shapes that were profiled as they are now.
MIB = float(1 << 20)
PROFILED_TRAFFIC = {
    "gemm2_kernel<128,128,2,4,A_KC,B_KC,bf16>": {"8192x4096x256+act": (20.2 + 128.1) * MIB, "3 x 8192x1024x256": (24.2 + 48.0) * MIB,
                                                 "8192x1024x256": (8.2 + 16.0) * MIB},
}


def kernel_roofline(rows):
    """Roofline object of the product kernel with the largest total time among the logged launches."""
    groups = {}
    for r in rows:
        groups.setdefault(r["kernel"], []).append(r)
    name, grp = max(groups.items(), key=lambda kv: sum(r["us"] for r in kv[1]))
    total_us = sum(r["us"] for r in grp)
    flops = nbytes = 0.0
    shapes = {}
    for r in grp:
        M, N, K, nb = r["M"], r["N"], r["K"], max(1, r.get("batch", 1))
        out_b = 4 if r["role"] in (5, 6) or "f32" in r["kernel"] else 2
        nbytes += nb * (2 * (M * K + N * K) + out_b * M * N + (2 * M * N if r["epilogue"] else 0))
        flops += 2.0 * M * N * K * nb
        key = (f"{nb} x " if nb > 1 else "") + f"{M}x{N}x{K}" + ("+act" if r["epilogue"] else "")
        shapes[key] = shapes.get(key, 0) + 1
    t_mfma, t_hbm = flops / (MFMA_BF16_PEAK_TFLOPS * 1e12), nbytes / (HBM_PEAK_GBS * 1e9)
    n = len(grp)
    if t_hbm >= t_mfma:
        ach = nbytes / (total_us * 1e-6) / 1e9
        roof = dict(bound="hbm", achieved=ach, peak=HBM_PEAK_GBS, unit="GB/s", frac=ach / HBM_PEAK_GBS)
    else:
        ach = flops / (total_us * 1e-6) / 1e12
        roof = dict(bound="mfma", achieved=ach, peak=MFMA_BF16_PEAK_TFLOPS, unit="TFLOP/s", frac=ach / MFMA_BF16_PEAK_TFLOPS)
    seen = PROFILED_TRAFFIC.get(name)
    traffic = None
    if seen and all(k in seen for k in shapes):
        traffic = sum(seen[k] * c for k, c in shapes.items()) / n
    roof.update(traffic=traffic, traffic_note="HBM bytes per launch from rocprofv3 FETCH_SIZE / WRITE_SIZE runs of this command, copy-calibrated "
                "(profiles/encoder_step_hbm_traffic.md, taken at commit d2842f5; csrc/mfma_gemm2.hip's kernel body is unchanged since); "
                "null when this kernel or its shapes were not the profiled ones", kernel=name, avg_us=total_us / n, launches=n, bytes_per_launch=nbytes / n, flops_per_launch=flops / n,
                share_of_logged_time=total_us / sum(r["us"] for r in rows), shapes=shapes,
                note="algorithmic bytes per launch = both operands read once + result written once (+ the activation tensor the "
                     "epilogue writes or reads); duration from HIP events on the launch stream around every launch of this kernel "
                     "in an eager pass over the timed steps")
    by_kernel = {k: dict(launches=len(v), total_us=sum(r["us"] for r in v)) for k, v in groups.items()}
    return roof, by_kernel


def graph_or_eager(torch, step_for_parity, steps, warmup, use_graph):
    if use_graph:
        return graph_timed(torch, step_for_parity, steps, warmup)
    return timed(torch, lambda s: step_for_parity(s & 1), steps, warmup)


def headline(args, torch, np, si, lrd):
    peaks = None if args.no_peaks else measure_peaks(torch, lrd)
    rank = lrd.quantize_rank(ENC_RANK, 64)
    deferred = not args.per_layer_backward
    enc = Encoder(lrd, torch, np, si, rank, seed_stream=0, deferred=deferred)
    masks = (lrd.freeze_mask(lrd.KIND_SVD, 0), lrd.freeze_mask(lrd.KIND_SVD, 1))

    def one(s):
        enc.step(masks[s & 1])

    for s in range(args.warmup):
        one(s)
    torch.cuda.synchronize()
    # eager pass over the K steps with every product bracketed by events (kernel-level roofline)
    per_step = 64 * ENC_LAYERS
    with lrd.ProfileLog(per_step * args.steps) as log:
        t0 = time.perf_counter()
        for s in range(args.steps):
            one(s)
        torch.cuda.synchronize()
        eager_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    rows = log.rows()
    roofline, by_kernel = kernel_roofline(rows)
    ms = eager_ms

    # The same K steps replayed from two captured HIP graphs (even / odd freeze mask): every kernel of the
    # step still runs, only the per-kernel launch gaps go.  Each replay is first checked bit for bit against
    # an eager step, with eager work between the replays.
    graph_ok = False
    if not args.no_graph:
        try:
            graphs = {}
            side = torch.cuda.Stream()
            for parity in (0, 1):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=side):
                    enc.step(masks[parity])
                graphs[parity] = g
            torch.cuda.synchronize()

            def snapshot():
                s = enc.st
                return [t.clone() for t in (enc.X[enc.n_layers], enc.G[0], s["up"]["dU"], s["up"]["dV"], s["dn"]["dU"], s["o"]["dV"],
                                            s["qkv"]["dU"], s["qkv"]["dU_by_member"], s["qkv"]["dV"])]

            graph_ok = True
            for rep in range(2):
                for parity in (0, 1):
                    one(parity)
                    torch.cuda.synchronize()
                    want = snapshot()
                    for t in (enc.X[enc.n_layers], enc.G[0]):
                        t.zero_()
                    graphs[parity].replay()
                    torch.cuda.synchronize()
                    got = snapshot()
                    # frozen factors' gradient buffers are not written in either mode, so all of them compare equal
                    graph_ok = graph_ok and all(torch.equal(a, b) for a, b in zip(want, got))
            if graph_ok:
                for s in range(args.warmup):
                    graphs[s & 1].replay()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for s in range(args.steps):
                    graphs[s & 1].replay()
                torch.cuda.synchronize()
                ms = (time.perf_counter() - t0) * 1e3 / args.steps
            del graphs
        except Exception as exc:      # capture unsupported: keep the eager figure
            print(f"bench.py: graph replay skipped ({exc})", file=sys.stderr)
            graph_ok = False

    n_even = (args.steps + 1) // 2
    flops = (enc.flops(masks[0]) * n_even + enc.flops(masks[1]) * (args.steps - n_even)) / args.steps
    roof = (enc.roof_us(masks[0]) * n_even + enc.roof_us(masks[1]) * (args.steps - n_even)) / args.steps
    tflops = flops / (ms * 1e-3) / 1e12
    out = dict(metric="decomposed-layer fwd+bwd throughput (12-layer encoder, hidden 1024, FFN 4096, SVD rank 256: Q/K/V/O and FFN linears)",
               value=tflops, unit="TFLOP/s", n_gpus=1, steps=args.steps, warmup=args.warmup, ms_per_step=ms,
               higher_is_better=True, scaling="weak", vs_baseline=None, dtype="bf16", data="synthetic",
               config=dict(workload="config 5: 12-layer transformer encoder, hidden 1024, 16 heads, FFN 4096, seq 512 x batch 16 = 8192 tokens, "
                                    "bf16; all Q/K/V/O and FFN linears SVD-decomposed at quantized rank 256, sequential freezing by step "
                                    "parity; decomposed-linear kernels only (attention, layer norm, residuals not run)",
                           backward="data gradients layer by layer, then the weight gradients of the 12 layers of each shape in one launch"
                                    if deferred else "one call per layer (data and weight gradients)",
                           tokens=ENC_T, rank=rank, layers=ENC_LAYERS, hidden=ENC_D, ffn=ENC_FF),
               tokens_per_s=ENC_T / (ms * 1e-3), frac_bf16_mfma_peak=tflops / MFMA_BF16_PEAK_TFLOPS,
               binding_roof=dict(roof_ms_per_step=roof * 1e-3, frac=roof * 1e-3 / ms,
                                 note="sum over the layer passes of max(flops / 2500 TFLOP/s, algorithmic bytes / 8000 GB/s), over the measured step"),
               launch="hip-graph replay" if graph_ok else "eager", eager_ms_per_step=eager_ms,
               roofline=roofline, kernels=by_kernel)
    if peaks is not None:
        out["peaks"] = peaks
    del enc
    torch.cuda.empty_cache()

    if not args.no_comparators:
        # Every comparator is timed the way the headline is (graph replay when that worked, else eager),
        # so the ratios compare GPU work and not host launch overhead.
        k = max(4, args.steps // 2)
        dense = DenseEncoder(lrd, torch, np, si)
        d_ms = graph_or_eager(torch, lambda parity: dense.step(), k, 2, graph_ok)
        d_tflops = dense.flops() / (d_ms * 1e-3) / 1e12
        del dense
        torch.cuda.empty_cache()
        raw_rank = rank + 1            # the paper's own example of an unquantized rank (257 -> 256), nothing frozen
        vanilla = Encoder(lrd, torch, np, si, raw_rank, seed_stream=1, grouped=False)
        v_ms = graph_or_eager(torch, lambda parity: vanilla.step(0), k, 2, graph_ok)
        del vanilla
        torch.cuda.empty_cache()
        unfrozen = Encoder(lrd, torch, np, si, rank, seed_stream=1)
        u_ms = graph_or_eager(torch, lambda parity: unfrozen.step(0), k, 2, graph_ok)
        del unfrozen
        torch.cuda.empty_cache()
        # the freezing ratio is taken between two runs on the headline's own schedule
        unfrozen = Encoder(lrd, torch, np, si, rank, seed_stream=1, deferred=deferred)
        ud_ms = graph_or_eager(torch, lambda parity: unfrozen.step(0), k, 2, graph_ok) if deferred else u_ms
        del unfrozen
        torch.cuda.empty_cache()
        per_layer = Encoder(lrd, torch, np, si, rank, seed_stream=0)
        pl_ms = graph_or_eager(torch, lambda parity: per_layer.step(masks[parity]), k, 2, graph_ok) if deferred else ms
        del per_layer
        torch.cuda.empty_cache()
        out["comparators"] = dict(dense_ms_per_step=d_ms, dense_tflops=d_tflops, dense_frac_bf16_mfma_peak=d_tflops / MFMA_BF16_PEAK_TFLOPS,
                                  speedup_vs_dense=d_ms / ms,
                                  vanilla_rank=raw_rank, vanilla_unfrozen_ms_per_step=v_ms, quantized_unfrozen_ms_per_step=u_ms,
                                  quantized_unfrozen_batched_wgrad_ms_per_step=ud_ms, frozen_per_layer_backward_ms_per_step=pl_ms,
                                  speedup_rank_quantization=v_ms / u_ms, speedup_freezing=ud_ms / ms, speedup_batched_wgrad=pl_ms / ms,
                                  speedup_combined=v_ms / ms,
                                  note="vanilla = raw rank 257 (Section 2.1's 257 -> 256 example), nothing frozen, Q/K/V as three separate layers, "
                                       "one backward call per layer; rank quantization compares it with rank 256 on that same per-layer schedule; "
                                       "freezing compares unfrozen and frozen on the headline's schedule; dense layers run their (large) weight "
                                       "gradients per layer; comparators are launched the same way as the headline (%s)"
                                       % ("hip-graph replay" if graph_ok else "eager"))
    if not args.no_workloads:
        out["workloads"] = other_workloads(args, torch, np, si, lrd, graph_ok)
    if not args.no_cpu_baseline:
        import oracle
        out["cpu_baseline"] = cpu_baseline(np, si, oracle, rank)
    return out


def other_workloads(args, torch, np, si, lrd, graph_ok):
    """The remaining workloads, each with time, TFLOP/s and fraction of its binding roof."""
    from paper_2309_03824_amd import factorize
    res = {}
    bf = torch.bfloat16
    k_steps = max(4, args.steps // 2)

    # ---- 12-block FFN stack, 768 -> 3072 -> 768, rank 192, 8192 tokens, sequential freezing
    rank2 = lrd.quantize_rank(int(0.25 * min(D_MODEL, D_FF)), 64)
    stack = Stack(lrd, torch, np, si, factorize, rank2, seed_stream=0, true_svd=False, deferred=True)
    masks = (lrd.freeze_mask(lrd.KIND_SVD, 0), lrd.freeze_mask(lrd.KIND_SVD, 1))
    ms2 = graph_or_eager(torch, lambda parity: stack.step(masks[parity]), k_steps, 2, graph_ok)
    stack.deferred = False
    ms2_per_layer = graph_or_eager(torch, lambda parity: stack.step(masks[parity]), k_steps, 2, graph_ok)
    fl2 = (stack.flops(masks[0]) + stack.flops(masks[1])) / 2
    roof2 = 0.0
    for mask in masks:
        for b in range(N_BLOCKS):
            for n_in, n_out, ao, ai, dx in ((D_MODEL, D_FF, True, False, b > 0), (D_FF, D_MODEL, False, True, True)):
                f, bw = layer_flops(T_TOKENS, n_in, n_out, rank2, mask, want_dx=dx)
                byf, byb = linear_bytes(T_TOKENS, n_in, n_out, rank2, mask, want_dx=dx, act_out=ao, act_in=ai)
                roof2 += roof_us(f + bw, byf + byb)[0] / 2
    del stack
    torch.cuda.empty_cache()
    res["ffn_stack_rank192"] = dict(workload="config 2: 12 x (768->3072, GELU, 3072->768), rank 192, 8192 tokens, sequential freezing; "
                                             "backward in two parts (batched weight gradients), the one-call-per-layer backward beside it",
                                    ms_per_step=ms2, per_layer_backward_ms_per_step=ms2_per_layer, tflops=fl2 / (ms2 * 1e-3) / 1e12, tokens_per_s=T_TOKENS / (ms2 * 1e-3),
                                    binding_roof_frac=roof2 * 1e-3 / ms2)

    # ---- one 4096 x 4096 layer, 16384 tokens: ranks 256 / 257 / 512 / 1024, first factor frozen, and the dense layer
    T, d = 16384, 4096
    gen = torch.Generator(device="cuda").manual_seed(230903824 + 3)

    def rnd(*shape, scale=1.0):
        return (torch.randn(*shape, device="cuda", generator=gen) * scale).to(bf)

    X, dY = rnd(T, d), rnd(T, d)
    Y, dX = torch.empty(T, d, dtype=bf, device="cuda"), torch.empty(T, d, dtype=bf, device="cuda")
    sweep = []
    for r in (256, 257, 512, 1024):
        V, U = rnd(r, d, scale=d ** -0.5), rnd(d, r, scale=r ** -0.5)
        H = torch.empty(T, r, dtype=bf, device="cuda")
        dV, dU = torch.empty(r, d, device="cuda"), torch.empty(d, r, device="cuda")
        ws = torch.empty(lrd.linear_workspace_bytes(T, d, d, r, lrd.BF16, 0) + 256, dtype=torch.uint8, device="cuda")
        fwd = event_us(torch, lambda: lrd.linear_fwd(X, V, U, None, Y, H, ws), 10)
        bwd = event_us(torch, lambda: lrd.linear_bwd(dY, X, H, V, U, dX, dV, dU, None, 1, ws), 10)
        f, b = layer_flops(T, d, d, r, 1)
        byf, byb = linear_bytes(T, d, d, r, 1)
        t_roof, bound = roof_us(f + b, byf + byb)
        sweep.append(dict(r=r, fwd_us=fwd, bwd_us_first_factor_frozen=bwd, tflops=(f + b) / ((fwd + bwd) * 1e-6) / 1e12,
                          frac_bf16_mfma_peak=(f + b) / ((fwd + bwd) * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                          binding_roof=bound, binding_roof_frac=t_roof / (fwd + bwd)))
        del V, U, H, dV, dU, ws
    W, dW = rnd(d, d, scale=d ** -0.5), torch.empty(d, d, device="cuda")
    wsd = torch.empty(lrd.dense_linear_workspace_bytes(T, d, d, lrd.BF16) + 256, dtype=torch.uint8, device="cuda")
    dense_f = event_us(torch, lambda: lrd.dense_linear_fwd(X, W, None, Y, wsd), 5)
    dense_b = event_us(torch, lambda: lrd.dense_linear_bwd(dY, X, W, dX, dW, wsd), 5)
    dense_tf = 6.0 * T * d * d / ((dense_f + dense_b) * 1e-6) / 1e12
    res["rank_sweep_4096"] = dict(workload="config 3: one 4096 x 4096 linear, 16384 tokens, fwd + bwd with the first factor frozen",
                                  ranks=sweep, dense=dict(fwd_us=dense_f, bwd_us=dense_b, tflops=dense_tf,
                                                          frac_bf16_mfma_peak=dense_tf / MFMA_BF16_PEAK_TFLOPS))
    del X, dY, Y, dX, W, dW, wsd
    torch.cuda.empty_cache()

    # ---- Tucker-2 3x3 stages, N = 128, ranks C/2, core frozen, and the dense layer
    stages = []
    N, k = 128, 3
    for C, hw in ((64, 56), (128, 28), (256, 14), (512, 7)):
        r = C // 2
        P = N * hw * hw
        g = lrd.conv_geom(N, hw, hw, C, C, r, r, k, 1, 1)
        Xc, dYc = rnd(N, hw, hw, C), rnd(N, hw, hw, C)
        Yc, dXc = torch.empty_like(Xc), torch.empty_like(Xc)
        P1, G, P2 = rnd(r, C, scale=C ** -0.5), rnd(r, k, k, r, scale=(k * k * r) ** -0.5), rnd(C, r, scale=r ** -0.5)
        A, B = torch.empty(N, hw, hw, r, dtype=bf, device="cuda"), torch.empty(N, hw, hw, r, dtype=bf, device="cuda")
        dP1, dG, dP2 = torch.empty(r, C, device="cuda"), torch.empty(r, k, k, r, device="cuda"), torch.empty(C, r, device="cuda")
        ws = torch.empty(lrd.tucker_conv_workspace_bytes(g, lrd.BF16, 0) + 256, dtype=torch.uint8, device="cuda")
        fwd = event_us(torch, lambda: lrd.tucker_conv_fwd(Xc, P1, G, P2, Yc, A, B, g, ws), 10)
        bwd = event_us(torch, lambda: lrd.tucker_conv_bwd(dYc, Xc, A, B, P1, G, P2, dXc, dP1, dG, dP2, 0b010, g, ws), 10)
        f_fwd = 2.0 * P * (C * r + k * k * r * r + r * C)
        f_bwd = 2.0 * f_fwd - 2.0 * P * k * k * r * r
        # algorithmic bytes, core frozen: X, Y, dY, dX once each; A, B written and read back; factors; fp32 1x1 gradients
        byts = 2.0 * (4 * P * C + 4 * P * r) + 2.0 * (2 * C * r + k * k * r * r) + 4.0 * 2 * C * r
        t_roof, bound = roof_us(f_fwd + f_bwd, byts)
        Wc, dWc = rnd(C, k, k, C, scale=(k * k * C) ** -0.5), torch.empty(C, k, k, C, device="cuda")
        wsd = torch.empty(lrd.dense_conv_workspace_bytes(g, lrd.BF16) + 256, dtype=torch.uint8, device="cuda")
        dfw = event_us(torch, lambda: lrd.dense_conv_fwd(Xc, Wc, Yc, g, wsd), 5)
        dbw = event_us(torch, lambda: lrd.dense_conv_bwd(dYc, Xc, Wc, dXc, dWc, g, wsd), 5)
        stages.append(dict(C=C, hw=hw, r=r, fwd_us=fwd, bwd_us_core_frozen=bwd, tflops=(f_fwd + f_bwd) / ((fwd + bwd) * 1e-6) / 1e12,
                           binding_roof=bound, binding_roof_frac=t_roof / (fwd + bwd), dense_fwd_us=dfw, dense_bwd_us=dbw,
                           speedup_vs_dense=(dfw + dbw) / (fwd + bwd)))
    res["tucker_stages"] = dict(workload="config 4: Tucker-2 3x3 stages, NHWC, N = 128, ranks C/2, fwd + bwd with the core frozen", stages=stages)

    # ---- the pair as two products (H through HBM: the default) against the LDS-staged fused pair, forward and data gradient
    pairs = []
    for T_, n_in, n_out, r in ((T_TOKENS, D_MODEL, D_FF, rank2), (ENC_T, ENC_D, ENC_FF, ENC_RANK), (ENC_T, ENC_D, ENC_D, ENC_RANK)):
        X, dY = rnd(T_, n_in), rnd(T_, n_out)
        V, U = rnd(r, n_in, scale=n_in ** -0.5), rnd(n_out, r, scale=r ** -0.5)
        Y, H, dX = torch.empty(T_, n_out, dtype=bf, device="cuda"), torch.empty(T_, r, dtype=bf, device="cuda"), torch.empty(T_, n_in, dtype=bf, device="cuda")
        ws = torch.empty(lrd.linear_workspace_bytes(T_, n_in, n_out, r, lrd.BF16, 3) + 256, dtype=torch.uint8, device="cuda")
        row = dict(tokens=T_, n_in=n_in, n_out=n_out, r=r)
        for name, mode in (("two_products", lrd.FUSION_NEVER), ("fused", lrd.FUSION_ALWAYS)):
            prev = lrd.set_fusion(mode)
            try:
                row[name + "_fwd_us"] = event_us(torch, lambda: lrd.linear_fwd(X, V, U, None, Y, H, ws), 8)
                row[name + "_dgrad_us"] = event_us(torch, lambda: lrd.linear_bwd(dY, X, H, V, U, dX, None, None, None, 3, ws), 8)
            finally:
                lrd.set_fusion(prev)
        pairs.append(row)
    res["fused_pair"] = dict(workload="one decomposed linear, forward (H saved) and data gradient (both factors frozen): two products with H / dH "
                                      "through HBM against one kernel that keeps them in LDS", pairs=pairs)
    return res


if __name__ == "__main__":
    main()
