"""GPU parity on the five workloads (shapes, dtypes and scalars of the five benchmark configurations), through the
C ABI, in the launch configuration bench.py times.

Coverage contract (what the oracle computed is what is claimed):
  C1  every element: norms (both paths), clip factors, sums, update with sigma = 0 and with sigma = 1, seed 0.
  C2, C3, C5  full-size micro-batch on the GPU; the oracle computes (a) the global norms of a sample of examples
      over the full manifest, (b) sampled entries of the clip-weighted sums of the full micro-batch (dense weights and
      biases, the first and last LayerNorm through both of its pass-2 paths, token-table entries of the most frequent
      ids, of ids that occur once and of random ids, position-table entries), with seeded stand-in norms fed to both
      sides, (c) every tensor for a leading subset of B' examples (GPU re-run at B'); embedding rows written are
      checked exactly at full size.
  C4  update over all ~334M parameters against the oracle on sampled slices (Philox words bit-exact on the same
      slices), gradient-SNR terms of all parameters against a chi-square bound / a library sum and, on the one-block
      manifest, against the oracle over every parameter; accumulation over micro-batches on a one-block manifest against the oracle; the FULL count
      (64 micro-batches of 1,024 examples, then the update with |B_t| = 65,536) on a width-reduced one-block manifest, every tensor and
      every parameter against the oracle; a B = 1024 dense layer with sampled entries; linearity of the accumulation on the GPU (an
      invariant, not oracle parity).
"""
import numpy as np
import pytest
import torch

import dp_synth as syn
from oracle import dp_oracle as orc

from gpu_util import DEV, assert_norms_close, assert_sums_close, f32_dev, host, to_dev

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2


def _layers(cfg_name, B=None, manifest=None, example_scale=None, seed_shift=0):
    cfg = syn.CONFIGS[cfg_name]
    man = manifest if manifest is not None else cfg["manifest"]()
    return cfg, man, syn.device_layer_inputs(man, B or cfg["B"], cfg["T"], dtype=cfg["dtype"], act_std=cfg["act_std"],
                                             grad_std=cfg["grad_std"], data_seed=cfg["data_seed"] + seed_shift, device=DEV,
                                             zipf_s=cfg.get("zipf_s", 1.1), example_scale=example_scale)


def _slice_layers(layers, n):
    out = []
    for l in layers:
        d = dict(l)
        for k in ("A", "G", "X", "ids", "H", "dL"):
            if k in d:
                d[k] = d[k][:n]
        out.append(d)
    return out


def _compare_all_tensors(run, man, sums_ref, tol, first=0):
    worst = 0.0
    for k, spec in enumerate(man):
        for j, (name, shp) in enumerate(spec.tensors()):
            got = host(run.view(run.S, first + k, j))
            worst = max(worst, assert_sums_close(got, sums_ref[k][j], tol, name))
    return worst


def _subset_parity(cfg_name, Bsub, C=None):
    """All tensors of the clip-weighted sum for the first Bsub examples, GPU re-run at B' = Bsub."""
    import paper_2108_01624_amd as pkg

    cfg, man, layers = _layers(cfg_name, B=Bsub)
    C = C or cfg["C"]
    with pkg.Context() as ctx:
        run = pkg.StepRunner(ctx, man, Bsub, device=DEV)
        n = run.pass1(layers)
        run.pass2(layers, C)
        ctx.sync()
        n_gpu = host(n)
        hl = syn.host_layer_slice(layers, range(Bsub))
        sums_ref, n_ref, c_ref = orc.microbatch_clip_sum(hl, C)
        assert_norms_close(n_gpu, n_ref, 1e-4, f"{cfg_name} norms")
        assert np.all(orc.clip_factors(n_gpu.astype(np.float64), C) ** 2 * n_ref <= C * C * (1 + 1e-3))
        worst = _compare_all_tensors(run, man, sums_ref, TOL_BF16)
        tok = [k for k, s in enumerate(man) if s.kind == "embedding" and not s.distinct]
        for k in tok:
            rows = np.nonzero(np.abs(host(run.view(run.S, k, 0))).sum(axis=1))[0]
            np.testing.assert_array_equal(rows, np.unique(hl[k]["ids"]))
    return worst


def _embedding_entries(l, S_E, ids_h, vs, c_ref, V, rng, name):
    """Entries (vs[j], ks[j]) of an embedding table's clip-weighted sum against the oracle's scatter over ALL examples,
    restricted to the sampled columns ks."""
    ks = rng.integers(0, S_E.shape[1], size=vs.size)
    Gc = l["G"][:, :, torch.as_tensor(ks, device=DEV)].float().cpu().numpy()
    ref = orc.clip_accumulate_embedding(ids_h, Gc, c_ref, V)[vs, np.arange(vs.size)]
    got = S_E[vs, ks].astype(np.float64)
    rms = np.sqrt(np.mean(ref ** 2))
    assert np.all(np.abs(got - ref) <= 1e-4 * (np.abs(ref) + rms)), (name, np.abs(got - ref).max(), rms)


def _full_size_parity(cfg_name, n_norm_samples=2, n_entries=24):
    """Full-size micro-batch on the GPU; sampled norms and sampled sum entries from the oracle."""
    import paper_2108_01624_amd as pkg

    cfg, man, layers = _layers(cfg_name)
    B, T, C = cfg["B"], cfg["T"], cfg["C"]
    rng = np.random.default_rng(cfg["data_seed"])
    with pkg.Context() as ctx:
        run = pkg.StepRunner(ctx, man, B, device=DEV)
        n = run.pass1(layers)
        ctx.sync()
        n_gpu = host(n).astype(np.float64)
        sample = sorted(set([0, B - 1] + list(rng.integers(0, B, size=n_norm_samples))))[: n_norm_samples + 2]
        n_ref = orc.microbatch_sqnorms(syn.host_layer_slice(layers, sample))
        assert_norms_close(n_gpu[sample], n_ref, 1e-4, f"{cfg_name} sampled global norms")
        assert np.isfinite(n_gpu).all() and (n_gpu > 0).all()

        # pass 2 at full size with seeded stand-in norms (both clip branches), sampled entries
        sq = syn.synthetic_sqnorms(B, C, cfg["data_seed"] + 5)
        c_ref = orc.clip_factors(sq.astype(np.float64), C)
        run.sqnorms[:B].copy_(f32_dev(sq))
        run.pass2(layers, C)
        ctx.sync()
        shapes_done = set()
        for k, (spec, l) in enumerate(zip(man, layers)):
            if spec.kind == "dense":
                if (spec.d_in, spec.d_out) in shapes_done and k % 7:
                    continue  # every shape, plus a scattering of layers
                shapes_done.add((spec.d_in, spec.d_out))
                ps = rng.integers(0, spec.d_in, size=n_entries)
                qs = rng.integers(0, spec.d_out, size=n_entries)
                ps[0], qs[0], ps[1], qs[1] = 0, 0, spec.d_in - 1, spec.d_out - 1
                Ac = l["A"][:, :, torch.as_tensor(ps, device=DEV)].float().cpu().numpy()
                Gc = l["G"][:, :, torch.as_tensor(qs, device=DEV)].float().cpu().numpy()
                ref = orc.clip_accumulate_dense_entries(Ac, Gc, c_ref)
                got = host(run.view(run.S, k, 0))[ps, qs].astype(np.float64)
                scale = np.sqrt(np.mean(ref ** 2))
                assert np.all(np.abs(got - ref) <= TOL_BF16 * (np.abs(ref) + scale)), (spec.name, np.abs(got - ref).max(), scale)
                assert np.linalg.norm(got - ref) <= 5e-3 * np.linalg.norm(ref), spec.name
                # bias: whole vector is cheap
                if spec.has_bias:
                    # the oracle's definition on a few columns, example by example
                    cols = qs[:8]
                    Gcol = l["G"][:, :, torch.as_tensor(cols, device=DEV)].float().cpu().numpy().astype(np.float64)
                    ref_b = sum(c_ref[i] * Gcol[i].sum(axis=0) for i in range(B))
                    got_b = host(run.view(run.S, k, 1))[cols].astype(np.float64)
                    sb = np.sqrt(np.mean(ref_b ** 2))
                    assert np.all(np.abs(got_b - ref_b) <= 1e-4 * (np.abs(ref_b) + sb)), spec.name
            elif spec.kind == "embedding" and not spec.distinct:
                S_E = host(run.view(run.S, k, 0))
                ids_h = host(l["ids"])
                rows = np.nonzero(np.abs(S_E).sum(axis=1))[0]
                np.testing.assert_array_equal(rows, np.unique(ids_h))
                # values: the oracle's scatter restricted to sampled columns, read at sampled rows - the most frequent
                # ids (their runs of sorted positions cross hundreds of 32-position chunks), ids that occur once, and
                # ids drawn from those present
                counts = np.bincount(ids_h.reshape(-1), minlength=spec.d_in)
                frequent = counts.argsort()[::-1][:6]
                once = np.nonzero(counts == 1)[0]
                present = np.nonzero(counts)[0]
                vs = np.concatenate([frequent, rng.choice(once, size=6, replace=False), rng.choice(present, size=12, replace=False)])
                assert counts[frequent[0]] > 32 * 100 and (counts[vs[6:12]] == 1).all()
                _embedding_entries(l, S_E, ids_h, vs, c_ref, spec.d_in, rng, spec.name)
            elif spec.kind == "embedding":
                S_E = host(run.view(run.S, k, 0))
                assert not S_E[T:].any()
                vs = np.concatenate([[0, T - 1], rng.integers(0, T, size=14)])
                _embedding_entries(l, S_E, host(l["ids"]), vs, c_ref, spec.d_in, rng, spec.name)
        # LayerNorm sums of the first and the last LayerNorm, sampled columns over all B examples: the sums pass 2 formed
        # from the per-example gradients that pass 1 kept, and the sums of the path that reads the inputs again
        ln = [k for k, spec in enumerate(man) if spec.kind == "layernorm"]
        for k in (ln[0], ln[-1]):
            l, d = layers[k], man[k].d_out
            cols = np.concatenate([[0, d - 1], rng.integers(0, d, size=14)])
            ct = torch.as_tensor(cols, device=DEV)
            ref_g, ref_b = orc.clip_accumulate_layernorm(l["X"][:, :, ct].float().cpu().numpy(),
                                                         l["G"][:, :, ct].float().cpu().numpy(), c_ref)
            again_g = torch.zeros(d, dtype=torch.float32, device=DEV)
            again_b = torch.zeros(d, dtype=torch.float32, device=DEV)
            ctx.clip_accumulate_layernorm_batched([l["X"]], [l["G"]], C, run.sqnorms[:B], [again_g], [again_b])
            ctx.sync()
            for what, got_g, got_b in (("kept", host(run.view(run.S, k, 0)), host(run.view(run.S, k, 1))),
                                       ("re-read", host(again_g), host(again_b))):
                for nm, got, ref in (("gamma", got_g[cols], ref_g), ("beta", got_b[cols], ref_b)):
                    rms = np.sqrt(np.mean(ref ** 2))
                    assert np.all(np.abs(got - ref) <= 1e-4 * (np.abs(ref) + rms)), (man[k].name, what, nm, np.abs(got - ref).max(), rms)


# ------------------------------------------------------------------------------------------------
# C1: single dense layer, fp32, every element
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("sigma,seed", [(0.0, 0), (1.0, 0)])
def test_c1_single_dense_fp32(dp, sigma, seed):
    import paper_2108_01624_amd as pkg

    cfg = syn.CONFIGS["C1"]
    B, T, C = cfg["B"], cfg["T"], cfg["C"]
    A = syn.normal_f32((B, T, 64), cfg["act_std"], cfg["data_seed"])
    G = syn.normal_f32((B, T, 64), cfg["grad_std"], cfg["data_seed"] + 1)
    W = syn.normal_f32((64 * 64,), 0.02, cfg["data_seed"] + 2)
    A_d, G_d = to_dev(A), to_dev(G)
    n_ref = orc.sqnorms_dense(A, G, False)
    for path in (pkg.DP_PATH_AUTO, pkg.DP_PATH_GRAM, pkg.DP_PATH_MATERIALISE):
        n = torch.zeros(B, dtype=torch.float32, device=DEV)
        dp.sqnorms_dense(A_d, G_d, False, path, n)
        dp.sync()
        assert_norms_close(host(n), n_ref, 1e-5, f"C1 norms path {path}")
    c_ref = orc.clip_factors(n_ref, C)
    assert (c_ref < 1).all()                       # with these distributions every example is clipped
    assert np.all(c_ref ** 2 * n_ref <= C * C * (1 + 1e-12))
    S = torch.zeros(64, 64, dtype=torch.float32, device=DEV)
    dp.clip_accumulate_dense(A_d, G_d, C, n, S, None)
    dp.sync()
    S_ref, _ = orc.clip_accumulate_dense(A, G, c_ref, False)
    assert_sums_close(host(S), S_ref, 1e-5, "C1 sum_W")
    S_host = host(S).reshape(-1).copy()
    th, m, v = f32_dev(W), torch.zeros(4096, dtype=torch.float32, device=DEV), torch.zeros(4096, dtype=torch.float32, device=DEV)
    kw = dict(sigma=sigma, C=C, seed=seed, step=1, batch_size=B, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-11, weight_decay=0.01)
    dp.noise_adamw(th, m, v, S.view(-1), **kw)
    dp.sync()
    th_ref, m_ref, v_ref, g_ref = orc.noise_adamw(W, np.zeros(4096), np.zeros(4096), S_host, elem_offset=0, **kw)
    np.testing.assert_allclose(host(m), m_ref, rtol=1e-5, atol=1e-6 * np.abs(m_ref).max())
    np.testing.assert_allclose(host(v), v_ref, rtol=2e-5, atol=1e-6 * np.abs(v_ref).max())
    assert np.all(np.abs(host(th) - th_ref) <= 1e-5 * np.abs(th_ref) + 1e-3 * 1e-3)
    if sigma > 0:
        w = torch.zeros(4096, dtype=torch.int32, device=DEV)
        dp.philox_u32(w, 0, seed, 1)
        dp.sync()
        np.testing.assert_array_equal(host(w).view(np.uint32), orc.philox_u32(4096, 0, seed, 1))
        # the gradient reconstructed from m carries the noise: g = m / (1 - beta1) at t = 1
        g_gpu = host(m).astype(np.float64) / (1 - float(np.float32(0.9)))
        np.testing.assert_allclose(g_gpu, g_ref, rtol=1e-4, atol=1e-6 * np.abs(g_ref).max())


# ------------------------------------------------------------------------------------------------
# C2, C3, C5
# ------------------------------------------------------------------------------------------------
def test_c2_bert_base_subset_all_tensors():
    worst = _subset_parity("C2", 4)
    assert worst < 5e-3, worst


def test_c2_bert_base_full_size_sampled():
    _full_size_parity("C2")


def test_c3_bert_large_subset_all_tensors():
    worst = _subset_parity("C3", 2)
    assert worst < 5e-3, worst


def test_c3_bert_large_full_size_sampled():
    _full_size_parity("C3")


def test_c3_mixed_clipping_both_branches():
    """Per-example gradient scales spread the norms around C: both branches of min(1, C/norm) occur."""
    import paper_2108_01624_amd as pkg

    Bsub = 6
    man = syn.bert_manifest(1, 1024, 4096, 30522, 512)
    scale = syn.example_scales(Bsub, 1e-4, 1.0, 77)
    cfg, man, layers = _layers("C3", B=Bsub, manifest=man, example_scale=scale)
    with pkg.Context() as ctx:
        run = pkg.StepRunner(ctx, man, Bsub, device=DEV)
        n = run.pass1(layers)
        ctx.sync()
        hl = syn.host_layer_slice(layers, range(Bsub))
        n_ref = orc.microbatch_sqnorms(hl)
        C = float(np.sqrt(np.median(n_ref)))
        run.pass2(layers, C)
        ctx.sync()
        sums_ref, _, c_ref = orc.microbatch_clip_sum(hl, C)
        assert (c_ref == 1).any() and (c_ref < 1).any()
        assert_norms_close(host(n), n_ref, 1e-4)
        _compare_all_tensors(run, man, sums_ref, TOL_BF16)


def test_c3_full_embedding_stage_all_tensors():
    """The embedding stage as Section 4.3 names it: word-piece, positional and token-type (2 rows) tables whose lookups are
    summed - one upstream gradient for all three - and the LayerNorm after the sum, in front of one BERT-Large block.
    Every tensor of the clip-weighted sum against the oracle through the step driver, both clip branches."""
    import paper_2108_01624_amd as pkg

    Bsub = 6
    man = syn.bert_manifest(1, 1024, 4096, 30522, 512, type_vocab=2)
    assert [s.name for s in man[:4]] == ["emb.tok", "emb.pos", "emb.type", "emb.ln"]
    assert syn.manifest_param_count(syn.bert_manifest(24, 1024, 4096, 30522, 512, type_vocab=2)) == 334_092_288
    scale = syn.example_scales(Bsub, 1e-4, 1.0, 78)
    cfg, man, layers = _layers("C3", B=Bsub, manifest=man, example_scale=scale)
    assert layers[0]["G"] is layers[1]["G"] and layers[1]["G"] is layers[2]["G"]      # one upstream gradient
    assert host(layers[2]["ids"])[0].tolist() == [0] * 64 + [1] * 64
    with pkg.Context() as ctx:
        run = pkg.StepRunner(ctx, man, Bsub, device=DEV)
        n = run.pass1(layers)
        ctx.sync()
        hl = syn.host_layer_slice(layers, range(Bsub))
        n_ref = orc.microbatch_sqnorms(hl)
        C = float(np.sqrt(np.median(n_ref)))
        run.pass2(layers, C)
        ctx.sync()
        sums_ref, _, c_ref = orc.microbatch_clip_sum(hl, C)
        assert (c_ref == 1).any() and (c_ref < 1).any()
        assert_norms_close(host(n), n_ref, 1e-4)
        _compare_all_tensors(run, man, sums_ref, TOL_BF16)
        # the token-type table: two rows, each the clip-weighted sum of its half of every sequence
        S_type = host(run.view(run.S, 2, 0)).astype(np.float64)
        assert S_type.shape == (2, 1024) and np.abs(S_type).min(axis=1).max() > 0
        assert_sums_close(S_type, sums_ref[2][0], 1e-4, "token-type table")
        assert_sums_close(host(run.view(run.S, 3, 0)), sums_ref[3][0], 1e-4, "embedding LayerNorm gain")


def test_c5_long_sequence_subset_all_tensors():
    worst = _subset_parity("C5", 2)
    assert worst < 5e-3, worst


def test_c5_gram_vs_materialise_each_shape():
    """T = 512: each path forced on each BERT-Large layer shape at the full micro-batch; they agree with each
    other on every example and with the oracle on sampled examples."""
    import paper_2108_01624_amd as pkg

    cfg = syn.CONFIGS["C5"]
    B, T = cfg["B"], cfg["T"]
    gen = torch.Generator(device=DEV)
    gen.manual_seed(cfg["data_seed"] + 11)
    with pkg.Context() as ctx:
        for d_in, d_out in ((1024, 1024), (1024, 4096), (4096, 1024)):
            A = (torch.randn(B, T, d_in, generator=gen, device=DEV)).to(torch.bfloat16)
            G = (torch.randn(B, T, d_out, generator=gen, device=DEV) * 1e-2).to(torch.bfloat16)
            res = {}
            for path in (pkg.DP_PATH_GRAM, pkg.DP_PATH_MATERIALISE):
                n = torch.zeros(B, dtype=torch.float32, device=DEV)
                ctx.sqnorms_dense(A, G, True, path, n)
                ctx.sync()
                res[path] = host(n).astype(np.float64)
            assert_norms_close(res[pkg.DP_PATH_GRAM], res[pkg.DP_PATH_MATERIALISE], 1e-4, f"{d_in}x{d_out} gram vs materialise")
            sample = [0, 57, B - 1]
            h = lambda t: t[sample].contiguous().cpu().view(torch.int16).numpy().view(np.uint16)
            ref = orc.sqnorms_dense(h(A), h(G), True)
            assert_norms_close(res[pkg.DP_PATH_GRAM][sample], ref, 1e-4, f"{d_in}x{d_out} gram vs oracle")
            assert_norms_close(res[pkg.DP_PATH_MATERIALISE][sample], ref, 1e-4, f"{d_in}x{d_out} materialise vs oracle")
            del A, G


def test_c5_long_sequence_full_size_sampled():
    _full_size_parity("C5", n_norm_samples=0, n_entries=16)


# ------------------------------------------------------------------------------------------------
# C4: mega-batch accumulation, noise, AdamW
# ------------------------------------------------------------------------------------------------
def test_c4_update_all_parameters_sampled_slices():
    import paper_2108_01624_amd as pkg

    cfg = syn.CONFIGS["C4"]
    P = syn.manifest_param_count(cfg["manifest"]())
    assert P == 334_088_192
    Bsz = cfg["B"] * cfg["micro_batches"]
    gen = torch.Generator(device=DEV)
    gen.manual_seed(cfg["data_seed"])
    th = torch.randn(P, generator=gen, device=DEV) * 0.02
    S = torch.randn(P, generator=gen, device=DEV) * 30.0
    m = torch.zeros(P, dtype=torch.float32, device=DEV)
    v = torch.zeros(P, dtype=torch.float32, device=DEV)
    rng = np.random.default_rng(4)
    L = 1 << 15
    offs = [0, P - L] + [int(x) for x in rng.integers(0, P - L, size=6)] + [4 * (2 ** 24) - 7]
    before = [(host(th[o:o + L]).copy(), host(S[o:o + L]).copy()) for o in offs]
    kw = dict(sigma=cfg["sigma"], C=cfg["C"], seed=cfg["noise_seed"], step=1, batch_size=Bsz, lr=cfg["lr"], beta1=cfg["beta1"],
              beta2=cfg["beta2"], eps=1e-11, weight_decay=cfg["weight_decay"])
    with pkg.Context() as ctx:
        # the variant that also returns the gradient-SNR terms (same update, bit for bit: see the kernel tests)
        S_sq = float((S.double() ** 2).sum().item())
        snr = torch.zeros(2, dtype=torch.float32, device=DEV)
        ctx.noise_adamw_snr(th, m, v, S, snr, zero_sum=True, **kw)
        ctx.sync()
        sig, noi = [float(x) for x in host(snr)]
        assert abs(sig - S_sq) <= 1e-5 * S_sq                      # a library reduction, not the oracle (size)
        sc2 = (float(np.float32(cfg["sigma"])) * float(np.float32(cfg["C"]))) ** 2
        assert abs(noi / sc2 - P) < 6 * np.sqrt(2.0 * P) + 1e-5 * P  # chi-square with P degrees of freedom
        w = torch.zeros(L, dtype=torch.int32, device=DEV)
        for o, (th0, S0) in zip(offs, before):
            ctx.philox_u32(w, o, cfg["noise_seed"], 1)
            ctx.sync()
            np.testing.assert_array_equal(host(w).view(np.uint32), orc.philox_u32(L, o, cfg["noise_seed"], 1))
            th_ref, m_ref, v_ref, g_ref = orc.noise_adamw(th0, np.zeros(L), np.zeros(L), S0, elem_offset=o, **kw)
            np.testing.assert_allclose(host(m[o:o + L]), m_ref, rtol=1e-5, atol=1e-6 * np.abs(m_ref).max())
            np.testing.assert_allclose(host(v[o:o + L]), v_ref, rtol=2e-5, atol=1e-6 * np.abs(v_ref).max())
            assert np.all(np.abs(host(th[o:o + L]) - th_ref) <= 1e-5 * np.abs(th_ref) + 1e-3 * cfg["lr"])
            assert not host(S[o:o + L]).any()
        # noise scale on the mean gradient: std of (g*Bsz - S)/(sigma*C) is 1
        o, (th0, S0) = offs[2], before[2]
        z = (host(m[o:o + L]).astype(np.float64) / (1 - float(np.float32(cfg["beta1"]))) * Bsz - S0) / (float(np.float32(cfg["sigma"])) * cfg["C"])
        assert abs(z.std() - 1) < 0.05 and abs(z.mean()) < 0.05


def test_c4_accumulation_over_micro_batches_one_block():
    """3 micro-batches of 8 examples accumulated into one sum buffer, then noise and the update."""
    import paper_2108_01624_amd as pkg

    cfg = syn.CONFIGS["C4"]
    man = syn.bert_manifest(1, 1024, 4096, 30522, 512)
    Bm, K = 8, 3
    with pkg.Context() as ctx:
        run = pkg.StepRunner(ctx, man, Bm, device=DEV)
        gen = torch.Generator(device=DEV)
        gen.manual_seed(5)
        run.theta.copy_(torch.randn(run.P, generator=gen, device=DEV) * 0.02)
        th0 = host(run.theta).copy()
        sums_ref = None
        for k in range(K):
            _, _, layers = _layers("C4", B=Bm, manifest=man, seed_shift=100 * k)
            run.pass1(layers)
            run.pass2(layers, cfg["C"])
            ctx.sync()
            sums_ref, _, _ = orc.microbatch_clip_sum(syn.host_layer_slice(layers, range(Bm)), cfg["C"], sums_ref)
        _compare_all_tensors(run, man, sums_ref, TOL_BF16)
        S_host = host(run.S).copy()
        kw = dict(sigma=cfg["sigma"], C=cfg["C"], seed=cfg["noise_seed"], step=1, batch_size=Bm * K, lr=cfg["lr"],
                  beta1=cfg["beta1"], beta2=cfg["beta2"], eps=1e-11, weight_decay=cfg["weight_decay"])
        snr = torch.zeros(2, dtype=torch.float32, device=DEV)
        run.update(snr_sq=snr, **kw)
        ctx.sync()
        # gradient-SNR terms over every parameter of the manifest, oracle in chunks
        sig = noi = 0.0
        for o in range(0, run.P, 1 << 22):
            a, b = orc.gradient_snr_terms(S_host[o:o + (1 << 22)], elem_offset=o, sigma=cfg["sigma"], C=cfg["C"],
                                          seed=cfg["noise_seed"], step=1)
            sig, noi = sig + a, noi + b
        np.testing.assert_allclose(host(snr), [sig, noi], rtol=1e-5)
        L = 1 << 16
        for o in (0, run.P - L, 31_000_000):
            th_ref, m_ref, _, _ = orc.noise_adamw(th0[o:o + L], np.zeros(L), np.zeros(L), S_host[o:o + L], elem_offset=o, **kw)
            np.testing.assert_allclose(host(run.m[o:o + L]), m_ref, rtol=1e-5, atol=1e-6 * np.abs(m_ref).max())
            assert np.all(np.abs(host(run.theta[o:o + L]) - th_ref) <= 1e-5 * np.abs(th_ref) + 1e-3 * cfg["lr"])
        assert not host(run.S).any()


def test_c4_full_count_64_micro_batches_of_1024_reduced_width():
    """The mega-batch at its FULL count - 64 micro-batches of 1,024 examples, 65,536 examples clip-accumulated into one sum
    buffer, then one noise + Adam step with |B_t| = 65,536 (Section 5.3) - on a width-reduced one-block manifest (hidden 128,
    FFN 512, T = 32, all three embedding tables and their LayerNorm) so that the oracle can materialise every one of the
    65,536 per-example gradients (about half a minute of host time).  Every tensor of the sum, then every parameter."""
    import paper_2108_01624_amd as pkg

    cfg = syn.CONFIGS["C4"]
    Bm, K, T = cfg["B"], cfg["micro_batches"], 32
    assert (Bm, K) == (1024, 64)
    man = syn.bert_manifest(1, 128, 512, vocab=512, max_pos=32, type_vocab=2)

    def batch(k):
        scale = syn.example_scales(Bm, 0.05, 20.0, 7000 + k)
        return syn.device_layer_inputs(man, Bm, T, dtype="bf16", act_std=1.0, grad_std=1e-2, data_seed=7100 + k, device=DEV,
                                       example_scale=scale)

    with pkg.Context() as ctx:
        run = pkg.StepRunner(ctx, man, Bm, device=DEV)
        run.theta.copy_(f32_dev(syn.normal_f32((run.P,), 0.02, 7001)))
        th0 = host(run.theta).astype(np.float64)
        C = float(np.sqrt(np.median(orc.microbatch_sqnorms(syn.host_layer_slice(batch(0), range(Bm))))))
        sums_ref, clipped, worst_norm = None, 0, 0.0
        for k in range(K):
            layers = batch(k)
            n = run.pass1(layers)
            run.pass2(layers, C)
            ctx.sync()
            sums_ref, n_ref, c_ref = orc.microbatch_clip_sum(syn.host_layer_slice(layers, range(Bm)), C, sums_ref)
            worst_norm = max(worst_norm, assert_norms_close(host(n), n_ref, 1e-4, f"micro-batch {k}"))
            clipped += int((c_ref < 1).sum())
        assert 0.2 * Bm * K < clipped < 0.8 * Bm * K          # both branches of the clip, in bulk
        _compare_all_tensors(run, man, sums_ref, TOL_BF16)
        S_ref = np.concatenate([x.reshape(-1) for s_ in sums_ref for x in s_])
        assert S_ref.shape[0] == run.P
        rel = np.linalg.norm(host(run.S) - S_ref) / np.linalg.norm(S_ref)
        assert rel < 5e-3, rel
        kw = dict(sigma=cfg["sigma"], C=C, seed=cfg["noise_seed"], step=1, batch_size=Bm * K, lr=cfg["lr"], beta1=cfg["beta1"],
                  beta2=cfg["beta2"], eps=1e-11, weight_decay=cfg["weight_decay"])
        S_gpu = host(run.S).copy()
        run.update(**kw)
        ctx.sync()
        # the update on the GPU's own sum (the sum itself was compared above): every parameter
        th_ref, m_ref, v_ref, g_ref = orc.noise_adamw(th0, np.zeros(run.P), np.zeros(run.P), S_gpu, elem_offset=0, **kw)
        np.testing.assert_allclose(host(run.m), m_ref, rtol=1e-5, atol=1e-6 * np.abs(m_ref).max())
        np.testing.assert_allclose(host(run.v), v_ref, rtol=2e-5, atol=1e-6 * np.abs(v_ref).max())
        assert np.all(np.abs(host(run.theta) - th_ref) <= 1e-5 * np.abs(th_ref) + 1e-3 * cfg["lr"])
        assert not host(run.S).any()
        # the noise is scaled by C / |B_t| on the mean gradient: per-coordinate std sigma * C / 65,536
        z = (host(run.m).astype(np.float64) / (1 - float(np.float32(cfg["beta1"]))) * (Bm * K) - S_gpu) / (float(np.float32(cfg["sigma"])) * float(np.float32(C)))
        assert abs(z.std() - 1) < 0.02 and abs(z.mean()) < 0.02


def test_c4_micro_batch_of_1024_dense_layer_and_linearity():
    """B = 1024 (131,072 token rows) on an FFN-shaped layer: sampled entries against the oracle; and
    S(batch 1 then batch 2) == S(batch 1) + S(batch 2) on the GPU (linearity of the accumulation)."""
    import paper_2108_01624_amd as pkg

    cfg = syn.CONFIGS["C4"]
    B, T, d_in, d_out, C = cfg["B"], cfg["T"], 1024, 4096, cfg["C"]
    gen = torch.Generator(device=DEV)
    gen.manual_seed(cfg["data_seed"] + 3)
    rng = np.random.default_rng(8)
    batches = []
    for k in range(2):
        A = torch.randn(B, T, d_in, generator=gen, device=DEV).to(torch.bfloat16)
        G = (torch.randn(B, T, d_out, generator=gen, device=DEV) * 1e-2).to(torch.bfloat16)
        sq = f32_dev(syn.synthetic_sqnorms(B, C, 90 + k))
        batches.append((A, G, sq))
    with pkg.Context() as ctx:
        single = []
        for A, G, sq in batches:
            S = torch.zeros(d_in, d_out, dtype=torch.float32, device=DEV)
            ctx.clip_accumulate_dense(A, G, C, sq, S, None)
            single.append(S)
        both = torch.zeros(d_in, d_out, dtype=torch.float32, device=DEV)
        for A, G, sq in batches:
            ctx.clip_accumulate_dense(A, G, C, sq, both, None)
        ctx.sync()
        lin = (single[0].double() + single[1].double()).cpu().numpy()
        assert_sums_close(host(both), lin, 1e-6, "linearity")
        A, G, sq = batches[0]
        ps, qs = rng.integers(0, d_in, size=16), rng.integers(0, d_out, size=16)
        Ac = A[:, :, torch.as_tensor(ps, device=DEV)].float().cpu().numpy()
        Gc = G[:, :, torch.as_tensor(qs, device=DEV)].float().cpu().numpy()
        ref = orc.clip_accumulate_dense_entries(Ac, Gc, orc.clip_factors(host(sq).astype(np.float64), C))
        got = host(single[0])[ps, qs].astype(np.float64)
        assert np.linalg.norm(got - ref) <= 5e-3 * np.linalg.norm(ref)


# ------------------------------------------------------------------------------------------------
# the token table tied to the output projection of the prediction slots
# ------------------------------------------------------------------------------------------------
def test_tied_output_projection_small_bert_all_tensors():
    """One block with position table and a token table that is also the output projection of 8 prediction slots:
    every tensor of the clip-weighted sum against the oracle, both clip branches."""
    import paper_2108_01624_amd as pkg

    B, T = 6, 48
    man = syn.bert_manifest(1, 256, 512, vocab=1000, max_pos=64, tied_pred=8)
    scale = np.array([30.0, 0.005, 30.0, 0.005, 1.0, 30.0], dtype=np.float32)
    layers = syn.device_layer_inputs(man, B, T, dtype="bf16", act_std=1.0, grad_std=1e-2, data_seed=4242, device=DEV,
                                     example_scale=scale)
    hl = syn.host_layer_slice(layers, range(B))
    sums_ref, n_ref, c_ref = orc.microbatch_clip_sum(hl, 1.0)
    assert (c_ref < 1).any() and (c_ref == 1).any()
    with pkg.Context() as ctx:
        run = pkg.StepRunner(ctx, man, B, device=DEV)
        n = run.pass1(layers)
        run.pass2(layers, 1.0)
        ctx.sync()
        assert_norms_close(host(n), n_ref, 1e-4, "norms with a tied table")
        _compare_all_tensors(run, man[1:], sums_ref[1:], TOL_BF16, first=1)
        # the tied table: a few rows (labels, frequent tokens) are orders of magnitude larger than the rest, and the
        # rounding of c*h to bf16 on the general GEMM path scales with the row, so entries are held against their row's rms
        got, ref = host(run.view(run.S, 0, 0)).astype(np.float64), sums_ref[0][0]
        assert np.linalg.norm(got - ref) <= 5e-3 * np.linalg.norm(ref)
        row_rms = np.sqrt((ref ** 2).mean(axis=1, keepdims=True))
        assert np.all(np.abs(got - ref) <= TOL_BF16 * (np.abs(ref) + row_rms)), np.abs(got - ref).max()
        # the tied layer alone: its norm is not the sum of its two uses
        tied = hl[0]
        assert tied["kind"] == "tied_embedding"
        whole = orc.sqnorms_tied_embedding(tied["ids"], tied["G"], tied["H"], tied["dL"])
        parts = orc.sqnorms_embedding(tied["ids"], tied["G"], tied["V"]) + orc.sqnorms_dense(tied["dL"], tied["H"], False)
        assert np.abs(whole - parts).max() > 1e-3 * whole.max()


def test_tied_output_projection_full_size_sampled():
    """BERT-Large word-piece table (30,522 rows padded to 30,528, width 1,024) tied to the output projection of 20
    prediction slots, B = 512, T = 128: norms of sampled examples and sampled entries of the sum from the oracle."""
    import paper_2108_01624_amd as pkg

    B, T, M, V, d, C = 512, 128, 20, 30528, 1024, 1.0
    man = [syn.LayerSpec("emb.tok", "tied_embedding", V, d, n_pred=M)]
    l = syn.device_layer_inputs(man, B, T, dtype="bf16", act_std=1.0, grad_std=1e-2, data_seed=5151, device=DEV)[0]
    rng = np.random.default_rng(5151)
    with pkg.Context() as ctx:
        n = torch.zeros(B, dtype=torch.float32, device=DEV)
        ctx.sqnorms_tied_embedding(l["ids"], l["G"], l["H"], l["dL"], n)
        ctx.sync()
        n_gpu = host(n).astype(np.float64)
        sample = [0, int(rng.integers(1, B - 1)), B - 1]
        hs = syn.host_layer_slice([l], sample)[0]
        n_ref = orc.sqnorms_tied_embedding(hs["ids"], hs["G"], hs["H"], hs["dL"])
        assert_norms_close(n_gpu[sample], n_ref, 1e-4, "tied table, sampled norms")
        assert np.isfinite(n_gpu).all() and (n_gpu > 0).all()

        sq = syn.synthetic_sqnorms(B, C, 5156)
        c_ref = orc.clip_factors(sq.astype(np.float64), C)
        S = torch.zeros(V, d, dtype=torch.float32, device=DEV)
        ctx.clip_accumulate_tied_embedding(l["ids"], l["G"], l["H"], l["dL"], C, f32_dev(sq), S)
        ctx.sync()
        ids_h = host(l["ids"])
        frequent = np.bincount(ids_h.reshape(-1), minlength=V).argsort()[::-1][:12]   # rows that the lookup writes too
        vs = np.concatenate([frequent, rng.integers(0, V, size=12)])
        ks = rng.integers(0, d, size=vs.size)
        kt = torch.as_tensor(ks, device=DEV)
        # output-projection part: a dense sum with input dL and output gradient H, entry (v, k)
        Ac = l["dL"][:, :, torch.as_tensor(vs, device=DEV)].float().cpu().numpy()
        Gc = l["H"][:, :, kt].float().cpu().numpy()
        ref = orc.clip_accumulate_dense_entries(Ac, Gc, c_ref)
        # lookup part: the scatter restricted to the sampled columns
        ref += orc.clip_accumulate_embedding(ids_h, l["G"][:, :, kt].float().cpu().numpy(), c_ref, V)[vs, np.arange(vs.size)]
        got = host(S)[vs, ks].astype(np.float64)
        scale = np.sqrt(np.mean(ref ** 2))
        assert np.all(np.abs(got - ref) <= TOL_BF16 * (np.abs(ref) + scale)), (np.abs(got - ref).max(), scale)
        assert np.linalg.norm(got - ref) <= 5e-3 * np.linalg.norm(ref)


def test_whole_step_is_reproducible_bit_for_bit():
    """Every reduction of the path has a fixed order (no atomics on floating point), so two runs of the same two-micro-batch
    step over a manifest with every layer kind (tied table, position table, LayerNorms, dense layers with shared inputs)
    give identical bits in the norms, the accumulated sum and the updated parameters."""
    import paper_2108_01624_amd as pkg

    B, T = 24, 64
    man = syn.bert_manifest(2, 256, 512, vocab=1024, max_pos=64, tied_pred=10)
    batches = [syn.device_layer_inputs(man, B, T, dtype="bf16", act_std=1.0, grad_std=1e-2, data_seed=6000 + k, device=DEV)
               for k in range(2)]
    for layers in batches:
        by_name = {l["name"]: l for l in layers}
        for name, l in by_name.items():
            if name.endswith(".k") or name.endswith(".v"):
                l["A"] = by_name[name[:-2] + ".q"]["A"]
    results = []
    for rep in range(2):
        with pkg.Context() as ctx:
            run = pkg.StepRunner(ctx, man, B, device=DEV)
            run.theta.copy_(f32_dev(syn.normal_f32((run.P,), 0.02, 6100)))
            norms = []
            for layers in batches:
                n = run.pass1(layers)
                ctx.sync()
                norms.append(host(n).copy())
                run.pass2(layers, 0.05)
            ctx.sync()
            S = host(run.S).copy()
            run.update(sigma=0.7, C=0.05, seed=77, step=1, batch_size=2 * B, lr=1e-3, beta1=0.9, beta2=0.999, weight_decay=0.01)
            ctx.sync()
            results.append((norms, S, host(run.theta).copy(), host(run.m).copy(), host(run.v).copy()))
    (n0, S0, th0, m0, v0), (n1, S1, th1, m1, v1) = results
    for a, b in zip(n0, n1):
        np.testing.assert_array_equal(a.view(np.uint32), b.view(np.uint32))
    for a, b in ((S0, S1), (th0, th1), (m0, m1), (v0, v1)):
        np.testing.assert_array_equal(a.view(np.uint32), b.view(np.uint32))
    assert np.abs(S0).max() > 0 and np.isfinite(th0).all()


# ------------------------------------------------------------------------------------------------
# schedule-driven steps: q_t micro-batches per step, eta_t per step, bias correction at t > 1
# ------------------------------------------------------------------------------------------------
def test_schedule_driven_steps_small_model():
    """Four steps of the whole path on a small BERT-shaped manifest: the number of micro-batches of step t comes
    from the increasing batch-size schedule, the learning rate from the warm-up / quadratic-decay schedule (both
    from the library's host entry points on the GPU side and from the oracle's own functions on the other), the
    state (theta, m, v) is carried from step to step on each side separately, mixed clipping."""
    import paper_2108_01624_amd as pkg

    man = syn.bert_manifest(1, 64, 128, 97, 32)
    Bm, T, C, steps = 8, 16, 0.05, 4
    sched = dict(b_start=8, b_end=24, ramp_steps=2, n_increments=2)
    lr_kw = dict(peak=2e-3, warmup_steps=2, total_steps=5)
    hp = dict(sigma=0.6, C=C, seed=77, beta1=0.9, beta2=0.999, eps=1e-11, weight_decay=0.5)
    with pkg.Context() as ctx:
        run = pkg.StepRunner(ctx, man, Bm, device=DEV)
        gen = torch.Generator(device=DEV)
        gen.manual_seed(6)
        run.theta.copy_(torch.randn(run.P, generator=gen, device=DEV) * 0.02)
        th = host(run.theta).astype(np.float64)
        m = np.zeros(run.P)
        v = np.zeros(run.P)
        seen = []
        well, lr_sum = np.ones(run.P, dtype=bool), 0.0
        for t in range(1, steps + 1):
            q_gpu = pkg.dp_batch_size_schedule(t, sched["b_start"], sched["b_end"], sched["ramp_steps"], sched["n_increments"])
            q_ref = orc.batch_size_schedule(t, **sched)
            lr_gpu = pkg.dp_lr_schedule(t, lr_kw["peak"], lr_kw["warmup_steps"], lr_kw["total_steps"])
            lr_ref = orc.lr_schedule(t, **lr_kw)
            assert q_gpu == q_ref and q_gpu % Bm == 0
            seen.append(q_gpu)
            sums_ref = None
            for k in range(q_gpu // Bm):
                scale = syn.example_scales(Bm, 0.05, 20.0, 100 * t + k)
                layers = syn.device_layer_inputs(man, Bm, T, dtype="bf16", act_std=1.0, grad_std=1e-2, data_seed=5000 + 100 * t + k,
                                                 device=DEV, example_scale=scale)
                n = run.pass1(layers)
                run.pass2(layers, C)
                ctx.sync()
                hl = syn.host_layer_slice(layers, range(Bm))
                sums_ref, n_ref, c_ref = orc.microbatch_clip_sum(hl, C, sums_ref)
                assert_norms_close(host(n), n_ref, 1e-4, f"step {t} micro-batch {k}")
                assert (c_ref < 1).any()
            _compare_all_tensors(run, man, sums_ref, TOL_BF16)
            S_ref = np.concatenate([x.reshape(-1) for s in sums_ref for x in s])
            assert S_ref.shape[0] == run.P
            run.update(step=t, batch_size=q_gpu, lr=lr_gpu, **hp)
            ctx.sync()
            th_prev = th
            th, m, v, g = orc.noise_adamw(th, m, v, S_ref, elem_offset=0, step=t, batch_size=q_ref, lr=lr_ref, **hp)
            np.testing.assert_allclose(host(run.m), m, rtol=1e-3, atol=2e-3 * np.abs(m).max())
            np.testing.assert_allclose(host(run.v), v, rtol=2e-3, atol=2e-3 * np.abs(v).max())
            # the Adam ratio mhat / sqrt(vhat) is +-1 at t = 1 and stays ill-conditioned where the gradient is within
            # the bf16 sum error of zero: the tight bound is asserted where |g| is well above that error (most
            # elements), the unconditional bound |ratio| <= 1 / sqrt(1 - beta2) scale everywhere
            err = np.abs(host(run.theta) - th)
            well &= np.abs(g) * q_ref > 0.05 * np.sqrt(np.mean(S_ref ** 2))    # errors are carried: well at EVERY step so far
            lr_sum += lr_ref
            assert well.mean() > 0.8
            assert np.all(err[well] <= 1e-5 * np.abs(th[well]) + 2e-2 * lr_sum), t
            assert np.all(err <= 1e-5 * np.abs(th) + 2.1 * lr_sum), t
            assert np.abs(th - th_prev).max() > 0.5 * lr_ref          # the step did move the parameters
        assert seen == [8, 16, 24, 24]
