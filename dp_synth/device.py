"""Seeded synthetic layer inputs generated directly in device memory (for full-size workloads that are
too large to draw on the host).  Harness code: random draws and dtype conversion only."""
from __future__ import annotations

import numpy as np

from .inputs import position_ids, segment_ids, zipf_ids


def _randn(shape, std, gen, dtype, device):
    import torch

    # drawn in fp32 chunk by chunk along dim 0, then rounded to the target dtype (RNE)
    out = torch.empty(shape, dtype=dtype, device=device)
    rows = shape[0]
    per = max(1, (1 << 27) // max(1, int(np.prod(shape[1:]))))
    for r0 in range(0, rows, per):
        r1 = min(rows, r0 + per)
        x = torch.randn((r1 - r0,) + tuple(shape[1:]), generator=gen, device=device, dtype=torch.float32)
        out[r0:r1] = (x * std).to(dtype)
    return out


def device_layer_inputs(manifest, B, T, *, dtype, act_std, grad_std, data_seed, device="cuda:0", zipf_s=1.1,
                        example_scale=None):
    """One dict per layer with device tensors: dense {A, G}, layernorm {X, G}, embedding {ids, G},
    tied_embedding {ids, G (gradient of the lookup output), H, dL}.
    `example_scale` (host fp32 [B]) multiplies example i's output gradients (mixed-clipping variant)."""
    import torch

    tdtype = torch.bfloat16 if dtype == "bf16" else torch.float32
    gen = torch.Generator(device=device)
    gen.manual_seed(int(data_seed))
    sc = None
    if example_scale is not None:
        sc = torch.from_numpy(np.asarray(example_scale, dtype=np.float32)).to(device)[:, None, None]
    layers = []
    group_grads = {}
    for k, spec in enumerate(manifest):
        d = dict(kind=spec.kind, name=spec.name, spec=spec)

        def grad(width):
            key = (spec.grad_group, width)
            if spec.grad_group and key in group_grads:
                return group_grads[key]   # the SAME tensor object: one upstream gradient for the whole group
            g = _randn((B, T, width), grad_std, gen, torch.float32 if sc is not None else tdtype, device)
            g = (g * sc).to(tdtype) if sc is not None else g
            if spec.grad_group:
                group_grads[key] = g
            return g

        if spec.kind == "dense":
            d["A"] = _randn((B, T, spec.d_in), act_std, gen, tdtype, device)
            d["G"] = grad(spec.d_out)
            d["has_bias"] = spec.has_bias
        elif spec.kind == "layernorm":
            d["X"] = _randn((B, T, spec.d_out), act_std, gen, tdtype, device)
            d["G"] = grad(spec.d_out)
        elif spec.kind == "tied_embedding":
            # lookup gradients as for an embedding; the output-projection side: inputs H like activations, logit
            # gradients dL dense and small with one large negative entry per used slot (the label's column, as in a
            # softmax cross-entropy gradient), labels drawn like token ids; each example uses between M/2 and M
            # of its M slots, the rows of the others are zero
            V, M = spec.d_in, spec.n_pred
            seed_k = int(data_seed) + 7919 * (k + 1)
            ids = zipf_ids(B, T, V, zipf_s, seed_k)
            d["ids"] = torch.from_numpy(ids).to(device)
            d["G"] = grad(spec.d_out)
            d["V"] = V
            d["H"] = _randn((B, M, spec.d_out), act_std, gen, tdtype, device)
            dL = _randn((B, M, V), grad_std / 8.0, gen, torch.float32, device)
            labels = torch.from_numpy(zipf_ids(B, M, V, zipf_s, seed_k + 1).astype(np.int64)).to(device)
            dL.scatter_add_(2, labels[:, :, None], torch.full((B, M, 1), -8.0 * grad_std, device=device))
            used = torch.from_numpy(np.random.default_rng(seed_k + 2).integers((M + 1) // 2, M + 1, size=B)).to(device)
            dL *= (torch.arange(M, device=device)[None, :] < used[:, None])[:, :, None]
            if sc is not None:
                dL *= sc
            d["dL"] = dL.to(tdtype)
        else:
            if spec.distinct:
                ids = position_ids(B, T)
            elif spec.segment:
                ids = segment_ids(B, T)
            else:
                ids = zipf_ids(B, T, spec.d_in, zipf_s, int(data_seed) + 7919 * (k + 1))
            d["ids"] = torch.from_numpy(ids).to(device)
            d["G"] = grad(spec.d_out)
            d["V"] = spec.d_in
            d["distinct"] = spec.distinct
        layers.append(d)
    return layers


def host_layer_slice(layers, examples):
    """Copy the given examples of every layer to the host in the form the oracle takes
    (bf16 as uint16 bit patterns, fp32 as float32, ids as int32)."""
    import torch

    idx = torch.as_tensor(list(examples), dtype=torch.long)

    def h(t):
        t = t[idx.to(t.device)].contiguous().cpu()
        if t.dtype == torch.bfloat16:
            return t.view(torch.int16).numpy().view(np.uint16)
        return t.numpy()

    out = []
    for l in layers:
        d = dict(kind=l["kind"])
        for key in ("A", "G", "X", "ids", "H", "dL"):
            if key in l:
                d[key] = h(l[key])
        if l["kind"] == "dense":
            d["has_bias"] = l["has_bias"]
        if l["kind"] in ("embedding", "tied_embedding"):
            d["V"] = l["V"]
        out.append(d)
    return out
