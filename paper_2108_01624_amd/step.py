"""Host-side step driver: walks a layer manifest and issues the C-ABI calls of one DP-SGD step
(Algorithm 1: per-example clip, sum over the micro-batch, accumulate over micro-batches, then noise
and the Adam update with decoupled weight decay).  Host logic only: every computation is a library call."""
from __future__ import annotations

from . import binding as B_


class StepRunner:
    """Owns the flat fp32 state (theta, m, v, clip-weighted sum S) of a manifest and the per-example
    squared-norm buffer.  Tensors of the flat space follow the manifest order (LayerSpec.tensors())."""

    def __init__(self, ctx, manifest, max_batch, device="cuda:0"):
        import torch

        self.ctx = ctx
        self.manifest = manifest
        self.offsets = []  # per layer: list of (offset, shape)
        off = 0
        for spec in manifest:
            cur = []
            for _, shp in spec.tensors():
                n = 1
                for s in shp:
                    n *= s
                off = (off + 3) // 4 * 4  # keep every tensor 16-byte aligned inside the flat buffers
                cur.append((off, shp))
                off += n
            self.offsets.append(cur)
        self.P = off
        self.S = torch.zeros(self.P, dtype=torch.float32, device=device)
        self.theta = torch.zeros(self.P, dtype=torch.float32, device=device)
        self.m = torch.zeros(self.P, dtype=torch.float32, device=device)
        self.v = torch.zeros(self.P, dtype=torch.float32, device=device)
        self.sqnorms = torch.zeros(max_batch, dtype=torch.float32, device=device)
        # per-example LayerNorm gradients kept from pass 1 for pass 2 (2 d floats per example and layer)
        self.max_batch = max_batch
        self.device = device
        self.ln_keep = {}
        self._kept_for = None

    def view(self, buf, layer, k):
        off, shp = self.offsets[layer][k]
        n = 1
        for s in shp:
            n *= s
        return buf[off:off + n].view(*shp)

    def _keep_buffer(self, k, d):
        """[max_batch, 2, d] floats for layer k of the manifest, allocated on first use."""
        import torch

        buf = self.ln_keep.get(k)
        if buf is None or buf.numel() < self.max_batch * 2 * d:
            buf = torch.empty(self.max_batch * 2 * d, dtype=torch.float32, device=self.device)
            self.ln_keep[k] = buf
        return buf

    @staticmethod
    def _ln_token(layers, nB):
        """Identifies the micro-batch whose LayerNorm gradients the keep buffers hold: batch size and input buffers."""
        return (nB, tuple((l["X"].data_ptr(), l["G"].data_ptr()) for l in layers if l["kind"] == "layernorm"))

    def pass1(self, layers, path=B_.DP_PATH_AUTO, batch_dense=True):
        """Per-example squared global norms of one micro-batch: sqnorms[:B] = sum over all layers.  The norm is a sum
        over layers, so dense layers of one shape, and LayerNorms of one shape, are handed over together."""
        ctx = self.ctx
        nB = layers[0]["G"].shape[0]
        n = self.sqnorms[:nB]
        ctx.zero_f32(n)
        groups, ln_groups = {}, {}
        for k, l in enumerate(layers):
            if l["kind"] == "dense":
                if batch_dense:
                    groups.setdefault((tuple(l["A"].shape), tuple(l["G"].shape), l["A"].dtype, bool(l["has_bias"])), []).append(l)
                else:
                    ctx.sqnorms_dense(l["A"], l["G"], l["has_bias"], path, n)
            elif l["kind"] == "layernorm":
                if batch_dense:
                    ln_groups.setdefault((tuple(l["X"].shape), l["X"].dtype), []).append(k)
                else:
                    ctx.sqnorms_layernorm(l["X"], l["G"], n)
            elif l["kind"] == "tied_embedding":   # lookup table that is also the output projection; G = dY
                ctx.sqnorms_tied_embedding(l["ids"], l["G"], l["H"], l["dL"], n)
            else:
                ctx.sqnorms_embedding(l["ids"], l["G"], l["V"], l["distinct"], n)
        self._kept_for = None
        for sel in ln_groups.values():
            Xs, Gs = [layers[k]["X"] for k in sel], [layers[k]["G"] for k in sel]
            d = Xs[0].shape[-1]
            if d % 4 == 0:
                ctx.sqnorms_layernorm_keep(Xs, Gs, n, [self._keep_buffer(k, d) for k in sel])
            else:
                ctx.sqnorms_layernorm_batched(Xs, Gs, n)
        if ln_groups and all(k[0][-1] % 4 == 0 for k in ln_groups):
            self._kept_for = self._ln_token(layers, nB)
        for key, ls in groups.items():
            # layers reading the very same input tensor (query / key / value projections) share its Gram matrix
            by_input = {}
            for l in ls:
                by_input.setdefault(l["A"].data_ptr(), []).append(l)
            shared = [v for v in by_input.values() if len(v) in (2, 3)] if path == B_.DP_PATH_AUTO else []
            for width in (3, 2):
                sel = [v for v in shared if len(v) == width]
                if sel:
                    ctx.sqnorms_dense_shared([v[0]["A"] for v in sel], [[l["G"] for l in v] for v in sel], key[3], n)
            taken = {id(l) for v in shared for l in v}
            rest = [l for l in ls if id(l) not in taken]
            if rest:
                ctx.sqnorms_dense_batched([l["A"] for l in rest], [l["G"] for l in rest], key[3], path, n)
        return n

    def pass2(self, layers, C, batch_dense=True):
        """S += sum_i clip(grad_i, C) for one micro-batch, using the norms left by pass1.  The sums of different
        layers are independent, so dense layers of one shape are handed over together (the library cuts them into launches that fill the chip)."""
        ctx = self.ctx
        nB = layers[0]["G"].shape[0]
        n = self.sqnorms[:nB]
        groups, ln_groups = {}, {}
        for k, l in enumerate(layers):
            if l["kind"] == "dense":
                if batch_dense:
                    groups.setdefault((tuple(l["A"].shape), tuple(l["G"].shape), l["A"].dtype), []).append(k)
                else:
                    sb = self.view(self.S, k, 1) if l["has_bias"] else None
                    ctx.clip_accumulate_dense(l["A"], l["G"], C, n, self.view(self.S, k, 0), sb)
            elif l["kind"] == "layernorm":
                if batch_dense:
                    ln_groups.setdefault((tuple(l["X"].shape), l["X"].dtype), []).append(k)
                else:
                    ctx.clip_accumulate_layernorm(l["X"], l["G"], C, n, self.view(self.S, k, 0), self.view(self.S, k, 1))
            elif l["kind"] == "tied_embedding":
                ctx.clip_accumulate_tied_embedding(l["ids"], l["G"], l["H"], l["dL"], C, n, self.view(self.S, k, 0))
            elif l.get("distinct"):
                ctx.clip_accumulate_positions(l["G"], C, n, self.view(self.S, k, 0))   # position ids: no sort needed
            else:
                ctx.clip_accumulate_embedding(l["ids"], l["G"], l["V"], C, n, self.view(self.S, k, 0))
        kept = self._kept_for is not None and self._kept_for == self._ln_token(layers, nB)   # pass 1 of this very micro-batch left the LayerNorm gradients behind
        for sel in ln_groups.values():
            sg, sb = [self.view(self.S, k, 0) for k in sel], [self.view(self.S, k, 1) for k in sel]
            if kept:
                d = layers[sel[0]]["X"].shape[-1]
                ctx.clip_accumulate_layernorm_kept([self.ln_keep[k] for k in sel], nB, d, C, n, sg, sb)
            else:
                ctx.clip_accumulate_layernorm_batched([layers[k]["X"] for k in sel], [layers[k]["G"] for k in sel], C, n, sg, sb)
        for sel in groups.values():
            ctx.clip_accumulate_dense_batched(
                [layers[k]["A"] for k in sel], [layers[k]["G"] for k in sel], C, n,
                [self.view(self.S, k, 0) for k in sel],
                [self.view(self.S, k, 1) if layers[k]["has_bias"] else None for k in sel])

    def update(self, *, sigma, C, seed, step, batch_size, lr, beta1, beta2, eps=1e-11, weight_decay, zero_sum=True,
               snr_sq=None):
        """Noise + Adam over the whole flat parameter space.  With `snr_sq` (a device tensor of two floats) the
        squared norms of the aggregated gradient and of the noise vector are written there (gradient-SNR terms)."""
        kw = dict(sigma=sigma, C=C, seed=seed, step=step, batch_size=batch_size, lr=lr, beta1=beta1, beta2=beta2, eps=eps,
                  weight_decay=weight_decay, zero_sum=zero_sum)
        if snr_sq is None:
            self.ctx.noise_adamw(self.theta, self.m, self.v, self.S, **kw)
        else:
            self.ctx.zero_f32(snr_sq, 2)
            self.ctx.noise_adamw_snr(self.theta, self.m, self.v, self.S, snr_sq, **kw)
