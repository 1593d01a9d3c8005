"""GPU parity tests: every entry point of the C ABI against the CPU oracle, element by element, on the
same seeded inputs, at sizes that span several tiles and a ragged tail.

Tolerances (derived in the design notes): Philox words and embedding indexing bit-exact; fp32 inputs
rel 1e-5 on norms and sums; bf16 inputs (fp32 accumulation) rel 2e-2, with the observed error printed
so that a regression to low-precision accumulation (~1e-2) is visible long before the bound."""
import numpy as np
import pytest
import torch

import dp_synth as syn
from oracle import dp_oracle as orc

from gpu_util import DEV, assert_norms_close, assert_sums_close, bf16_dev, f32_dev, host, to_dev

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-5
TOL_BF16 = 2e-2


def gen(shape, std, seed, dtype):
    return syn.normal_bf16_bits(shape, std, seed) if dtype == "bf16" else syn.normal_f32(shape, std, seed)


def tol_of(dtype):
    return TOL_BF16 if dtype == "bf16" else TOL_F32


# ------------------------------------------------------------------------------------------------
# Philox stream and normals
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("off,n,seed,step", [(0, 4096, 0, 1), (1, 1000, 1234, 1), (5, 3, 7, 2), (4 * 2 ** 32 - 6, 50, 99, 3),
                                             (123456789012, 777, 2 ** 63 + 11, 2 ** 32 + 9), (0, 1, 5, 1), (3, 1, 5, 1)])
def test_philox_words_bit_exact(dp, off, n, seed, step):
    import paper_2108_01624_amd as pkg

    out = torch.zeros(n, dtype=torch.int32, device=DEV)
    dp.philox_u32(out, off, seed, step)
    dp.sync()
    got = host(out).view(np.uint32)
    np.testing.assert_array_equal(got, orc.philox_u32(n, off, seed, step))


def test_philox_empty(dp):
    out = torch.zeros(4, dtype=torch.int32, device=DEV)
    dp.philox_u32(out, 0, 1, 1, n=0)
    dp.sync()
    assert host(out).tolist() == [0, 0, 0, 0]


@pytest.mark.parametrize("off,n", [(0, 1 << 16), (3, 1001)])
def test_normals_match_oracle(dp, off, n):
    out = torch.zeros(n, dtype=torch.float32, device=DEV)
    dp.normal_f32(out, off, 1234, 1)
    dp.sync()
    z = host(out).astype(np.float64)
    ref = orc.normals(n, off, 1234, 1)
    # fp32 log / sqrt / sincos against fp64: |z| <= 5.8, a few ulp of fp32
    assert np.abs(z - ref).max() < 1e-5, np.abs(z - ref).max()


def test_normals_full_u_range(dp):
    """Scan many blocks and check the extreme uniforms (u near 0 and near 1), where log is most delicate."""
    n = 1 << 22
    out = torch.zeros(n, dtype=torch.float32, device=DEV)
    dp.normal_f32(out, 0, 42, 1)
    dp.sync()
    z = host(out).astype(np.float64)
    ref = orc.normals(n, 0, 42, 1)
    assert np.abs(z - ref).max() < 1e-5
    assert np.isfinite(z).all()


# ------------------------------------------------------------------------------------------------
# noise + AdamW
# ------------------------------------------------------------------------------------------------
def _adam_case(dp, n, off, sigma, seed, step, steps=1, zero_sum=False, batch=32, lr=1e-3, b1=0.9, b2=0.999, wd=0.01, C=1.0,
               misalign=0):
    th0 = syn.normal_f32((n,), 0.02, 50)
    pad = misalign
    th = f32_dev(np.concatenate([np.zeros(pad, np.float32), th0]))[pad:]
    m = torch.zeros(n + pad, dtype=torch.float32, device=DEV)[pad:]
    v = torch.zeros(n + pad, dtype=torch.float32, device=DEV)[pad:]
    r_th, r_m, r_v = th0.astype(np.float64), np.zeros(n), np.zeros(n)
    for k in range(steps):
        S = syn.normal_f32((n,), 3.0, 60 + k)
        S_d = f32_dev(np.concatenate([np.zeros(pad, np.float32), S]))[pad:]
        dp.noise_adamw(th, m, v, S_d, n=n, elem_offset=off, sigma=sigma, C=C, seed=seed, step=step + k, batch_size=batch,
                       lr=lr, beta1=b1, beta2=b2, eps=1e-11, weight_decay=wd, zero_sum=zero_sum)
        dp.sync()
        r_th, r_m, r_v, g = orc.noise_adamw(r_th.astype(np.float32), r_m.astype(np.float32), r_v.astype(np.float32), S,
                                            elem_offset=off, sigma=sigma, C=C, seed=seed, step=step + k, batch_size=batch,
                                            lr=lr, beta1=b1, beta2=b2, eps=1e-11, weight_decay=wd)
        # the oracle restarts each step from the fp32 state the GPU holds, so errors do not compound
        gm, gv, gth = host(m).astype(np.float64), host(v).astype(np.float64), host(th).astype(np.float64)
        np.testing.assert_allclose(gm, r_m, rtol=1e-5, atol=1e-6 * np.abs(r_m).max())
        np.testing.assert_allclose(gv, r_v, rtol=2e-5, atol=1e-6 * np.abs(r_v).max())
        # the Adam term is bounded by lr and ill-conditioned where g ~ 0
        assert np.all(np.abs(gth - r_th) <= 1e-5 * np.abs(r_th) + 1e-3 * lr), np.abs(gth - r_th).max()
        if zero_sum:
            assert not host(S_d).any()
        else:
            np.testing.assert_array_equal(host(S_d), S)
        r_th, r_m, r_v = gth, gm, gv
    return gth


def test_adamw_c1_sigma0(dp):
    _adam_case(dp, 64 * 64, 0, 0.0, 0, 1)


def test_adamw_c1_sigma1_seed0(dp):
    _adam_case(dp, 64 * 64, 0, 1.0, 0, 1)


@pytest.mark.parametrize("n,off,misalign", [(1, 0, 0), (3, 0, 0), (4099, 0, 0), (1000, 5, 0), (1000, 4, 1), (7, 2, 3),
                                            (100003, 8, 0)])
def test_adamw_ragged_and_offset(dp, n, off, misalign):
    _adam_case(dp, n, off, 0.6, 1234, 1, misalign=misalign)


def test_adamw_multi_step_and_zero_sum(dp):
    _adam_case(dp, 5000, 0, 0.6, 1234, 1, steps=4, zero_sum=True, b1=0.75, b2=0.9, wd=1.0, lr=6.0902e-4, C=3.2429e-3)


def test_adamw_slicing_invariance(dp):
    """The noise depends on the global element index only: updating two slices equals updating the whole."""
    n = 10007
    th0 = syn.normal_f32((n,), 0.02, 70)
    S = syn.normal_f32((n,), 3.0, 71)
    kw = dict(sigma=0.6, C=1.0, seed=9, step=3, batch_size=64, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-11, weight_decay=0.5)
    res = []
    for cut in (None, 4000, 4001):
        th, m, v, S_d = f32_dev(th0), torch.zeros(n, dtype=torch.float32, device=DEV), torch.zeros(n, dtype=torch.float32, device=DEV), f32_dev(S)
        if cut is None:
            dp.noise_adamw(th, m, v, S_d, elem_offset=100, **kw)
        else:
            dp.noise_adamw(th[:cut], m[:cut], v[:cut], S_d[:cut], n=cut, elem_offset=100, **kw)
            dp.noise_adamw(th[cut:], m[cut:], v[cut:], S_d[cut:], n=n - cut, elem_offset=100 + cut, **kw)
        dp.sync()
        res.append((host(th), host(m), host(v)))
    for r in res[1:]:
        for a, b in zip(res[0], r):
            np.testing.assert_array_equal(a, b)


def test_adamw_untouched_row_is_pure_decay(dp):
    n = 256
    th0 = syn.normal_f32((n,), 0.02, 72)
    th, m, v, S = f32_dev(th0), torch.zeros(n, dtype=torch.float32, device=DEV), torch.zeros(n, dtype=torch.float32, device=DEV), torch.zeros(n, dtype=torch.float32, device=DEV)
    dp.noise_adamw(th, m, v, S, sigma=0.0, C=1.0, seed=0, step=1, batch_size=8, lr=1e-3, beta1=0.9, beta2=0.999,
                   eps=1e-11, weight_decay=0.5)
    dp.sync()
    np.testing.assert_allclose(host(th), th0.astype(np.float64) * (1 - float(np.float32(1e-3)) * 0.5), rtol=2e-7)
    assert not host(m).any() and not host(v).any()


# ------------------------------------------------------------------------------------------------
# gradient signal-to-noise terms fused into the update (Section 5.2.1)
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("n,off,sigma,zero_sum", [(64 * 64, 0, 1.0, False), (1, 0, 0.6, False), (4099, 0, 0.6, True),
                                                   (1000, 5, 0.6, False), (7, 2, 0.0, False), (300007, 8, 0.6, True),
                                                   (1 << 20, 0, 0.6, False)])
def test_noise_adamw_snr_matches_oracle_and_plain_update(dp, n, off, sigma, zero_sum):
    th0 = syn.normal_f32((n,), 0.02, 80)
    S = syn.normal_f32((n,), 3.0, 81)
    kw = dict(elem_offset=off, sigma=sigma, C=0.7, seed=1234, step=2, batch_size=64, lr=1e-3, beta1=0.9, beta2=0.999,
              eps=1e-11, weight_decay=0.5)
    z = lambda: torch.zeros(n, dtype=torch.float32, device=DEV)
    th_a, m_a, v_a, S_a = f32_dev(th0), z(), z(), f32_dev(S)
    th_b, m_b, v_b, S_b = f32_dev(th0), z(), z(), f32_dev(S)
    snr = torch.full((2,), 7.0, dtype=torch.float32, device=DEV)     # "+=": a stale value must survive as an offset
    dp.noise_adamw(th_a, m_a, v_a, S_a, zero_sum=zero_sum, **kw)
    dp.noise_adamw_snr(th_b, m_b, v_b, S_b, snr, zero_sum=zero_sum, **kw)
    dp.sync()
    for a, b in ((th_a, th_b), (m_a, m_b), (v_a, v_b), (S_a, S_b)):   # the update itself is bit-identical
        np.testing.assert_array_equal(host(a), host(b))
    sig, noi = orc.gradient_snr_terms(S, elem_offset=off, sigma=sigma, C=0.7, seed=1234, step=2)
    got = host(snr).astype(np.float64) - 7.0
    assert abs(got[0] - sig) <= 1e-5 * sig + 1e-5, (got[0], sig)
    assert abs(got[1] - noi) <= 1e-5 * noi + 1e-5, (got[1], noi)
    if sigma == 0.0:
        assert got[1] == 0.0


def test_noise_adamw_snr_slices_add_and_repeat_exactly(dp):
    n, off, cut = 50021, 12, 20001
    S = syn.normal_f32((n,), 2.0, 82)
    kw = dict(sigma=0.6, C=1.0, seed=5, step=1, batch_size=32, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-11, weight_decay=0.0)
    z = lambda k: torch.zeros(k, dtype=torch.float32, device=DEV)
    out = []
    for rep in range(2):
        whole, parts = z(2), z(2)
        dp.noise_adamw_snr(z(n), z(n), z(n), f32_dev(S), whole, elem_offset=off, **kw)
        S_d = f32_dev(S)
        dp.noise_adamw_snr(z(cut), z(cut), z(cut), S_d[:cut], parts, n=cut, elem_offset=off, **kw)
        dp.noise_adamw_snr(z(n - cut), z(n - cut), z(n - cut), S_d[cut:], parts, n=n - cut, elem_offset=off + cut, **kw)
        dp.sync()
        out.append((host(whole), host(parts)))
    np.testing.assert_allclose(out[0][0], out[0][1], rtol=1e-5)
    np.testing.assert_array_equal(out[0][0], out[1][0])   # fixed summation order: reproducible bit for bit
    np.testing.assert_array_equal(out[0][1], out[1][1])
    sig, noi = orc.gradient_snr_terms(S, elem_offset=off, sigma=0.6, C=1.0, seed=5, step=1)
    np.testing.assert_allclose(out[0][0], [sig, noi], rtol=1e-5)


# ------------------------------------------------------------------------------------------------
# dense layers: norms
# ------------------------------------------------------------------------------------------------
DENSE_SHAPES = [
    # dtype, B, T, d_in, d_out
    ("f32", 32, 16, 64, 64),      # the single-dense-layer workload
    ("f32", 3, 5, 7, 6),          # ragged everything
    ("f32", 2, 33, 20, 12),
    ("bf16", 5, 128, 256, 384),   # one Gram block, big GEMM tiles
    ("bf16", 3, 100, 72, 136),    # ragged T and widths
    ("bf16", 2, 16, 64, 64),      # T far below one block
    ("bf16", 9, 300, 264, 128),   # 3 x 3 Gram blocks with a ragged last block, 9 examples over 8 XCD lanes
    ("bf16", 2, 512, 128, 1024),  # 4 x 4 Gram cells: two diagonal blocks and two row pairs
    ("bf16", 1, 1, 8, 8),         # T = 1
    ("bf16", 3, 300, 128, 192),   # 3 x 3 cells, ragged last one: a diagonal block, the last diagonal cell leading a row pair, a lone cell
    ("bf16", 2, 129, 64, 64),     # one row into the second block
    ("bf16", 11, 256, 320, 64),   # 2 x 2 cells = one diagonal block per example, 11 examples over the 8 XCD lanes
    ("bf16", 4, 20, 1032, 72),    # T <= 32: the one-tile kernel, widths that end inside a 128-column chunk
    ("bf16", 3, 32, 520, 256),    # T = 32 exactly
    ("bf16", 2, 33, 128, 64),     # one row more: back to the 128-row kernels
    ("bf16", 5, 20, 1984, 192),   # T <= 32, widths multiples of 64: the ring-fed one-tile kernel, more stages than the ring holds
    ("bf16", 3, 32, 64, 128),     # ... and fewer
    ("bf16", 2, 640, 64, 128),    # 5 x 5 Gram cells: units of every kind, among them an off-diagonal cell on its own
    ("bf16", 9, 1100, 64, 64),    # 9 x 9 cells with a ragged last one: the cells of the unpaired last panel form row pairs of their own
    ("bf16", 1, 2100, 64, 64),    # 17 x 17 cells: past the unit kernel's table, the register-staged kernel's block pairs
    ("bf16", 2, 2048, 64, 128),   # 16 x 16 cells: the unit kernel's largest plane (8 diagonal blocks + 56 row pairs)
]


@pytest.mark.parametrize("dtype,B,T,d_in,d_out", DENSE_SHAPES)
@pytest.mark.parametrize("has_bias", [False, True])
def test_sqnorms_dense_paths(dp, dtype, B, T, d_in, d_out, has_bias):
    import paper_2108_01624_amd as pkg

    A = gen((B, T, d_in), 1.0, 100, dtype)
    G = gen((B, T, d_out), 0.1, 101, dtype)
    ref = orc.sqnorms_dense(A, G, has_bias)
    A_d, G_d = to_dev(A), to_dev(G)
    errs = {}
    for path in (pkg.DP_PATH_GRAM, pkg.DP_PATH_MATERIALISE, pkg.DP_PATH_AUTO):
        n = torch.zeros(B, dtype=torch.float32, device=DEV)
        dp.sqnorms_dense(A_d, G_d, has_bias, path, n)
        dp.sync()
        errs[path] = assert_norms_close(host(n), ref, tol_of(dtype), f"path {path}")
    if dtype == "bf16":
        # fp32 accumulation of exact bf16 products: the real error is ~1e-6, far inside the 2e-2 bound
        assert max(errs.values()) < 1e-4, errs


def test_sqnorms_accumulate_over_layers(dp):
    """Each call ADDS to sqnorms: two layers in sequence give the sum of both contributions."""
    import paper_2108_01624_amd as pkg

    B, T = 4, 128
    A1, G1 = gen((B, T, 64), 1.0, 110, "bf16"), gen((B, T, 128), 0.1, 111, "bf16")
    A2, G2 = gen((B, T, 128), 1.0, 112, "bf16"), gen((B, T, 64), 0.1, 113, "bf16")
    n = torch.zeros(B, dtype=torch.float32, device=DEV)
    dp.sqnorms_dense(to_dev(A1), to_dev(G1), True, pkg.DP_PATH_GRAM, n)
    dp.sqnorms_dense(to_dev(A2), to_dev(G2), False, pkg.DP_PATH_MATERIALISE, n)
    dp.sync()
    ref = orc.sqnorms_dense(A1, G1, True) + orc.sqnorms_dense(A2, G2, False)
    assert_norms_close(host(n), ref, 1e-4)


# ------------------------------------------------------------------------------------------------
# dense layers: clip-weighted sums
# ------------------------------------------------------------------------------------------------
ACC_SHAPES = [
    ("f32", 32, 16, 64, 64),
    ("f32", 3, 5, 7, 6),
    ("f32", 4, 40, 70, 130),
    ("bf16", 8, 128, 256, 384),    # 256 x 256 tiles, ragged second tile column, split over rows
    ("bf16", 6, 96, 72, 136),      # 128 x 128 tiles, ragged
    ("bf16", 64, 128, 256, 256),   # 8192 rows: several XCD-interleaved splits
    ("bf16", 3, 50, 512, 264),     # rows not a multiple of the staged tile height
    ("bf16", 2, 7, 8, 8),
    ("bf16", 5, 128, 256, 256),    # 5 examples over 3 row splits (2 + 2 + 1 whole examples)
    ("bf16", 7, 64, 256, 512),     # two stages per example: every stage starts or ends one
    ("bf16", 3, 192, 320, 256),    # six stages per example, ragged tile row
]


@pytest.mark.parametrize("dtype,B,T,d_in,d_out", ACC_SHAPES)
def test_clip_accumulate_dense(dp, dtype, B, T, d_in, d_out):
    A = gen((B, T, d_in), 1.0, 120, dtype)
    G = gen((B, T, d_out), 0.1, 121, dtype)
    C = 1.0
    sq = syn.synthetic_sqnorms(B, C, 122)           # both clip branches occur
    c = orc.clip_factors(sq.astype(np.float64), C)
    assert (c == 1).any() and (c < 1).any() or B < 3
    SW_ref, Sb_ref = orc.clip_accumulate_dense(A, G, c, True)
    init_W = syn.normal_f32((d_in, d_out), float(np.abs(SW_ref).mean()), 123)   # the call must ADD to the buffer
    init_b = syn.normal_f32((d_out,), float(np.abs(Sb_ref).mean()), 124)
    S_W, S_b = f32_dev(init_W), f32_dev(init_b)
    dp.clip_accumulate_dense(to_dev(A), to_dev(G), C, f32_dev(sq), S_W, S_b)
    dp.sync()
    rel = assert_sums_close(host(S_W) - init_W.astype(np.float64), SW_ref, tol_of(dtype) + 1e-6, "sum_W")
    assert_sums_close(host(S_b) - init_b.astype(np.float64), Sb_ref, tol_of(dtype) + 1e-6, "sum_b")
    if dtype == "bf16":
        assert rel < 5e-3, rel  # re-rounding c*g to bf16 costs ~2^-9 per term, averaged over the sum


def test_clip_accumulate_dense_noop_clip_is_flat_gemm(dp):
    """With no example clipped the bf16 path multiplies by 1 exactly: the result is the plain A^T G."""
    B, T, d_in, d_out = 4, 64, 128, 128
    A, G = gen((B, T, d_in), 1.0, 130, "bf16"), gen((B, T, d_out), 0.1, 131, "bf16")
    sq = np.full(B, 1e-6, np.float32)
    S_W = torch.zeros(d_in, d_out, dtype=torch.float32, device=DEV)
    dp.clip_accumulate_dense(to_dev(A), to_dev(G), 1.0, f32_dev(sq), S_W, None)
    dp.sync()
    ref, _ = orc.clip_accumulate_dense(A, G, np.ones(B), False)
    assert_sums_close(host(S_W), ref, 1e-5, "unclipped sum")


def test_clip_factors(dp):
    sq = np.array([0.0, 1e-12, 0.25, 1.0, 4.0, 1e12], np.float32)
    c = torch.zeros(6, dtype=torch.float32, device=DEV)
    dp.clip_factors(f32_dev(sq), 1.0, c)
    dp.sync()
    np.testing.assert_allclose(host(c), orc.clip_factors(sq.astype(np.float64), 1.0), rtol=1e-6)
    assert host(c)[0] == 1.0 and host(c)[3] == 1.0


def test_dense_pipeline_clip_invariant_and_determinism(dp):
    """Norms from pass 1 feed pass 2; c_i^2 n_i <= C^2; a second run gives the same bits."""
    import paper_2108_01624_amd as pkg

    B, T, d_in, d_out = 16, 128, 256, 256
    scale = syn.example_scales(B, 1e-3, 1.0, 140)
    A = gen((B, T, d_in), 1.0, 141, "bf16")
    G = syn.f32_to_bf16_bits(syn.normal_f32((B, T, d_out), 1e-2, 142) * scale[:, None, None])
    A_d, G_d = to_dev(A), to_dev(G)
    n_ref = orc.sqnorms_dense(A, G, True)
    C = float(np.sqrt(np.median(n_ref)))
    c_ref = orc.clip_factors(n_ref, C)
    assert (c_ref == 1).any() and (c_ref < 1).any()
    outs = []
    for _ in range(2):
        n = torch.zeros(B, dtype=torch.float32, device=DEV)
        S_W, S_b = torch.zeros(d_in, d_out, dtype=torch.float32, device=DEV), torch.zeros(d_out, dtype=torch.float32, device=DEV)
        dp.sqnorms_dense(A_d, G_d, True, pkg.DP_PATH_AUTO, n)
        dp.clip_accumulate_dense(A_d, G_d, C, n, S_W, S_b)
        c = torch.zeros(B, dtype=torch.float32, device=DEV)
        dp.clip_factors(n, C, c)
        dp.sync()
        outs.append((host(n), host(S_W), host(S_b), host(c)))
    for a, b in zip(*outs):
        np.testing.assert_array_equal(a, b)
    n, S_W, S_b, c = outs[0]
    assert_norms_close(n, n_ref, 1e-4)
    assert np.all(c.astype(np.float64) ** 2 * n <= C * C * (1 + 1e-5))
    SW_ref, Sb_ref = orc.clip_accumulate_dense(A, G, c_ref, True)
    assert_sums_close(S_W, SW_ref, TOL_BF16, "sum_W")
    assert_sums_close(S_b, Sb_ref, TOL_BF16, "sum_b")


@pytest.mark.parametrize("T", [128, 48])  # 128: operands straight into LDS, accumulators rescaled at example boundaries;
                                          # 48: register-staged kernel, clip factor applied to the staged rows
def test_dense_one_example_with_a_huge_norm(dp, T):
    """Finite inputs, one example whose gradient norm is 5e18 (its squared norm, 2.5e37, is near the top of the fp32 range)
    between neighbours with norms around 1: its clip factor is 2e-19, the ratios of neighbouring factors 5e18 and 2e-19, and
    every path must still give the oracle's sums."""
    import paper_2108_01624_amd as pkg

    B, d_in, d_out, C, big = 6, 256, 256, 1.0, 3
    A = gen((B, T, d_in), 1.0, 150, "bf16")
    Gf = syn.normal_f32((B, T, d_out), 1e-2, 151)
    n0 = orc.sqnorms_dense(A, syn.f32_to_bf16_bits(Gf), True)
    Gf /= np.sqrt(n0)[:, None, None].astype(np.float32)          # every example: norm ~1
    Gf[big] *= np.float32(5e18)
    G = syn.f32_to_bf16_bits(Gf)
    n_ref = orc.sqnorms_dense(A, G, True)
    assert 1e37 < n_ref[big] < 3e38 and n_ref[big - 1] < 4 and n_ref[big + 1] < 4
    c_ref = orc.clip_factors(n_ref, C)
    SW_ref, Sb_ref = orc.clip_accumulate_dense(A, G, c_ref, True)
    A_d, G_d = to_dev(A), to_dev(G)
    n = torch.zeros(B, dtype=torch.float32, device=DEV)
    S_W, S_b = torch.zeros(d_in, d_out, dtype=torch.float32, device=DEV), torch.zeros(d_out, dtype=torch.float32, device=DEV)
    dp.sqnorms_dense(A_d, G_d, True, pkg.DP_PATH_GRAM, n)
    dp.clip_accumulate_dense(A_d, G_d, C, n, S_W, S_b)
    dp.sync()
    assert_norms_close(host(n), n_ref, 1e-4, "norms")
    assert_sums_close(host(S_W), SW_ref, TOL_BF16, "sum_W")
    assert_sums_close(host(S_b), Sb_ref, TOL_BF16, "sum_b")
    # the clipped example still weighs as much as a neighbour: dropping it would be seen
    SW_without, _ = orc.clip_accumulate_dense(np.delete(A, big, 0), np.delete(G, big, 0), np.delete(c_ref, big), True)
    assert np.linalg.norm(SW_ref - SW_without) > 0.1 * np.linalg.norm(SW_ref)


@pytest.mark.parametrize("T", [128, 48])
@pytest.mark.parametrize("bad", [np.inf, np.nan])
def test_dense_non_finite_norm_poisons_the_sum_and_is_reported(dp, T, bad):
    """A squared norm that overflowed fp32 (or is NaN) has no clip factor: every path alike turns the sums it enters
    into NaN, and dp_sync reports DP_ERR_VALUE once."""
    import paper_2108_01624_amd as pkg

    B, d_in, d_out = 4, 256, 256
    A, G = gen((B, T, d_in), 1.0, 152, "bf16"), gen((B, T, d_out), 1e-2, 153, "bf16")
    sq = np.array([0.5, 2.0, bad, 3.0], np.float32)
    S_W, S_b = torch.zeros(d_in, d_out, dtype=torch.float32, device=DEV), torch.zeros(d_out, dtype=torch.float32, device=DEV)
    dp.clip_accumulate_dense(to_dev(A), to_dev(G), 1.0, f32_dev(sq), S_W, S_b)
    with pytest.raises(pkg.DpError) as e:
        dp.sync()
    assert e.value.status == -5
    dp.sync()  # the error word is cleared
    assert np.isnan(host(S_W)).all() and np.isnan(host(S_b)).all()
    c = torch.zeros(B, dtype=torch.float32, device=DEV)
    dp.clip_factors(f32_dev(sq), 1.0, c)
    with pytest.raises(pkg.DpError):
        dp.sync()
    got = host(c)
    assert np.isnan(got[2]) and np.isfinite(got[[0, 1, 3]]).all()


# ------------------------------------------------------------------------------------------------
# LayerNorm
# ------------------------------------------------------------------------------------------------
LN_SHAPES = [("f32", 32, 16, 64), ("f32", 3, 5, 6), ("f32", 2, 9, 260), ("bf16", 6, 128, 768), ("bf16", 3, 100, 1024),
             ("bf16", 2, 17, 8), ("bf16", 40, 128, 264)]


@pytest.mark.parametrize("dtype,B,T,d", LN_SHAPES)
def test_layernorm_norms_and_sums(dp, dtype, B, T, d):
    X = gen((B, T, d), 1.0, 150, dtype)
    G = gen((B, T, d), 0.1, 151, dtype)
    X_d, G_d = to_dev(X), to_dev(G)
    n = f32_dev(np.full(B, 0.5, np.float32))
    dp.sqnorms_layernorm(X_d, G_d, n)
    dp.sync()
    assert_norms_close(host(n).astype(np.float64) - 0.5, orc.sqnorms_layernorm(X, G), 1e-5 if dtype == "f32" else 1e-4)
    C = 1.0
    sq = syn.synthetic_sqnorms(B, C, 152)
    c = orc.clip_factors(sq.astype(np.float64), C)
    Sg_ref, Sb_ref = orc.clip_accumulate_layernorm(X, G, c)
    S_g, S_b = torch.ones(d, dtype=torch.float32, device=DEV), torch.ones(d, dtype=torch.float32, device=DEV)
    dp.clip_accumulate_layernorm(X_d, G_d, C, f32_dev(sq), S_g, S_b)
    dp.sync()
    t = 1e-5 if dtype == "f32" else 1e-4
    assert_sums_close(host(S_g).astype(np.float64) - 1.0, Sg_ref, t, "sum_gamma")
    assert_sums_close(host(S_b).astype(np.float64) - 1.0, Sb_ref, t, "sum_beta")


@pytest.mark.parametrize("dtype,n,B,T,d", [("bf16", 3, 9, 128, 1024), ("bf16", 19, 4, 33, 264), ("f32", 2, 5, 17, 20), ("bf16", 1, 3, 8, 64),
                                          ("f32", 17, 2, 9, 6)])
def test_layernorm_batched(dp, dtype, n, B, T, d):
    """Several LayerNorms of one shape in one call (more than one launch's worth at n > 16): each layer against the oracle,
    the norms against the sum over layers."""
    Xs = [gen((B, T, d), 1.0, 900 + l, dtype) for l in range(n)]
    Gs = [gen((B, T, d), 0.1 * (1 + l % 3), 950 + l, dtype) for l in range(n)]
    Xd, Gd = [to_dev(x) for x in Xs], [to_dev(g) for g in Gs]
    nrm = f32_dev(np.full(B, 0.25, np.float32))
    dp.sqnorms_layernorm_batched(Xd, Gd, nrm)
    dp.sync()
    ref = sum(orc.sqnorms_layernorm(x, g) for x, g in zip(Xs, Gs))
    assert_norms_close(host(nrm).astype(np.float64) - 0.25, ref, 1e-5 if dtype == "f32" else 1e-4, "batched LN norms")
    C = 1.0
    sq = syn.synthetic_sqnorms(B, C, 990)
    c = orc.clip_factors(sq.astype(np.float64), C)
    Sg = [torch.full((d,), 2.0, dtype=torch.float32, device=DEV) for _ in range(n)]
    Sb = [torch.full((d,), -1.0, dtype=torch.float32, device=DEV) for _ in range(n)]
    dp.clip_accumulate_layernorm_batched(Xd, Gd, C, f32_dev(sq), Sg, Sb)
    dp.sync()
    t = 1e-5 if dtype == "f32" else 1e-4
    for l in range(n):
        g_ref, b_ref = orc.clip_accumulate_layernorm(Xs[l], Gs[l], c)
        assert_sums_close(host(Sg[l]).astype(np.float64) - 2.0, g_ref, t, f"layer {l} sum_gamma")
        assert_sums_close(host(Sb[l]).astype(np.float64) + 1.0, b_ref, t, f"layer {l} sum_beta")
    if d % 4:
        return
    # the same through kept per-example gradients: pass 1 writes them, pass 2 only weights and adds them
    keep = [torch.full((B, 2, d), 7.0, dtype=torch.float32, device=DEV) for _ in range(n)]
    nrm2 = f32_dev(np.full(B, 0.25, np.float32))
    dp.sqnorms_layernorm_keep(Xd, Gd, nrm2, keep)
    dp.sync()
    np.testing.assert_array_equal(host(nrm2), host(nrm))                   # same kernel, same order: same bits
    for l in (0, n - 1):
        for i in (0, B - 1):
            gg, gb = orc.layernorm_example_grads(Xs[l][i], Gs[l][i])
            k = host(keep[l][i]).astype(np.float64)
            np.testing.assert_allclose(k[0], gg, rtol=t, atol=t * np.abs(gg).max())
            np.testing.assert_allclose(k[1], gb, rtol=t, atol=t * np.abs(gb).max())
    Sg2 = [torch.full((d,), 2.0, dtype=torch.float32, device=DEV) for _ in range(n)]
    Sb2 = [torch.full((d,), -1.0, dtype=torch.float32, device=DEV) for _ in range(n)]
    dp.clip_accumulate_layernorm_kept(keep, B, d, C, f32_dev(sq), Sg2, Sb2)
    dp.sync()
    for l in range(n):
        g_ref, b_ref = orc.clip_accumulate_layernorm(Xs[l], Gs[l], c)
        assert_sums_close(host(Sg2[l]).astype(np.float64) - 2.0, g_ref, t, f"layer {l} sum_gamma from kept gradients")
        assert_sums_close(host(Sb2[l]).astype(np.float64) + 1.0, b_ref, t, f"layer {l} sum_beta from kept gradients")


# ------------------------------------------------------------------------------------------------
# embeddings
# ------------------------------------------------------------------------------------------------
EMB_SHAPES = [("f32", 6, 20, 4, 13), ("f32", 3, 7, 6, 11), ("bf16", 8, 128, 1024, 30522), ("bf16", 5, 100, 264, 300),
              ("bf16", 70, 128, 64, 50), ("bf16", 3, 512, 256, 1000)]


@pytest.mark.parametrize("dtype,B,T,d,V", EMB_SHAPES)
def test_embedding_norms_and_sums(dp, dtype, B, T, d, V):
    ids = syn.zipf_ids(B, T, V, 1.1, 160)
    G = gen((B, T, d), 0.1, 161, dtype)
    ids_d, G_d = to_dev(ids), to_dev(G)
    n = torch.zeros(B, dtype=torch.float32, device=DEV)
    dp.sqnorms_embedding(ids_d, G_d, V, False, n)
    dp.sync()
    assert_norms_close(host(n), orc.sqnorms_embedding(ids, G, V), 1e-5 if dtype == "f32" else 1e-4, "token norms")
    C = 1.0
    sq = syn.synthetic_sqnorms(B, C, 162)
    c = orc.clip_factors(sq.astype(np.float64), C)
    ref = orc.clip_accumulate_embedding(ids, G, c, V)
    S = torch.zeros(V, d, dtype=torch.float32, device=DEV)
    dp.clip_accumulate_embedding(ids_d, G_d, V, C, f32_dev(sq), S)
    dp.sync()
    got = host(S)
    # indexing is exact: the rows written are exactly the ids present
    np.testing.assert_array_equal(np.nonzero(np.abs(got).sum(axis=1))[0], np.unique(ids))
    assert_sums_close(got, ref, 1e-5 if dtype == "f32" else 1e-4, "sum_E")
    # a second micro-batch accumulates on top
    dp.clip_accumulate_embedding(ids_d, G_d, V, C, f32_dev(sq), S)
    dp.sync()
    assert_sums_close(host(S), 2 * ref, 1e-5 if dtype == "f32" else 1e-4, "sum_E twice")


@pytest.mark.parametrize("B,T,V", [(8, 128, 30522), (70, 128, 5), (3, 1000, 2), (1, 1, 1)])
def test_embedding_counts_are_exact(dp, B, T, V):
    """All-ones gradients and no clipping: sum_E[v, :] is the count of v (small integers, exact in fp32)."""
    d = 8
    ids = syn.zipf_ids(B, T, V, 1.1, 170)
    G = syn.f32_to_bf16_bits(np.ones((B, T, d), np.float32))
    S = torch.zeros(V, d, dtype=torch.float32, device=DEV)
    dp.clip_accumulate_embedding(to_dev(ids), to_dev(G), V, 1.0, f32_dev(np.full(B, 1e-9, np.float32)), S)
    n = torch.zeros(B, dtype=torch.float32, device=DEV)
    dp.sqnorms_embedding(to_dev(ids), to_dev(G), V, False, n)
    dp.sync()
    cnt = np.bincount(ids.reshape(-1), minlength=V).astype(np.float32)
    np.testing.assert_array_equal(host(S), np.repeat(cnt[:, None], d, axis=1))
    ref_n = np.array([d * float((np.bincount(r, minlength=V).astype(np.float64) ** 2).sum()) for r in ids])
    np.testing.assert_array_equal(host(n).astype(np.float64), ref_n)


@pytest.mark.parametrize("dtype,B,T,d", [("bf16", 6, 128, 1024), ("f32", 4, 9, 5), ("bf16", 300, 16, 64)])
def test_position_embedding(dp, dtype, B, T, d):
    V = T + 3
    ids = syn.position_ids(B, T)
    G = gen((B, T, d), 0.1, 180, dtype)
    n = torch.zeros(B, dtype=torch.float32, device=DEV)
    dp.sqnorms_embedding(to_dev(ids), to_dev(G), V, True, n)
    n2 = torch.zeros(B, dtype=torch.float32, device=DEV)
    dp.sqnorms_embedding(to_dev(ids), to_dev(G), V, False, n2)   # the general path agrees on distinct ids
    dp.sync()
    ref = orc.sqnorms_embedding(ids, G, V)
    t = 1e-5 if dtype == "f32" else 1e-4
    assert_norms_close(host(n), ref, t)
    assert_norms_close(host(n2), ref, t)
    sq = syn.synthetic_sqnorms(B, 1.0, 181)
    c = orc.clip_factors(sq.astype(np.float64), 1.0)
    S = torch.zeros(V, d, dtype=torch.float32, device=DEV)
    dp.clip_accumulate_embedding(to_dev(ids), to_dev(G), V, 1.0, f32_dev(sq), S)
    dp.sync()
    got = host(S)
    assert not got[T:].any()
    assert_sums_close(got, orc.clip_accumulate_embedding(ids, G, c, V), t, "sum_pos")


def test_embedding_out_of_range_id_is_reported(dp):
    import paper_2108_01624_amd as pkg

    B, T, d, V = 2, 8, 8, 10
    ids = syn.zipf_ids(B, T, V, 1.1, 190)
    ids[1, 3] = V
    G = gen((B, T, d), 0.1, 191, "bf16")
    n = torch.zeros(B, dtype=torch.float32, device=DEV)
    dp.sqnorms_embedding(to_dev(ids), to_dev(G), V, False, n)
    with pytest.raises(pkg.DpError) as e:
        dp.sync()
    assert e.value.status == -6
    dp.sync()  # the error word is cleared
    ids[1, 3] = -1
    S = torch.zeros(V, d, dtype=torch.float32, device=DEV)
    dp.clip_accumulate_embedding(to_dev(ids), to_dev(G), V, 1.0, f32_dev(np.ones(B, np.float32)), S)
    with pytest.raises(pkg.DpError):
        dp.sync()
    # the valid tokens were still accumulated, the bad one skipped
    ids_ok = ids.copy()
    got = host(S)
    ref = np.zeros((V, d))
    Gf = orc.to_f64(G)
    for i in range(B):
        for t in range(T):
            if 0 <= ids_ok[i, t] < V:
                ref[ids_ok[i, t]] += Gf[i, t]
    assert_sums_close(got, ref, 1e-5)


# ------------------------------------------------------------------------------------------------
# argument errors (host side: nothing is launched)
# ------------------------------------------------------------------------------------------------
def test_argument_errors(dp):
    import paper_2108_01624_amd as pkg

    lib = pkg.load_library()
    h = dp.handle
    x = torch.zeros(64, dtype=torch.float32, device=DEV)
    p = x.data_ptr()
    assert lib.dp_sqnorms_dense(h, None, p, 0, 1, 1, 4, 4, 0, 0, p) == -1
    assert lib.dp_sqnorms_dense(h, p, p, 7, 1, 1, 4, 4, 0, 0, p) == -3
    assert lib.dp_sqnorms_dense(h, p, p, 0, 1, 1, 4, 4, 0, 9, p) == -3
    assert lib.dp_sqnorms_dense(h, p, p, 0, -1, 1, 4, 4, 0, 0, p) == -2
    assert lib.dp_sqnorms_dense(h, p, p, 1, 1, 1, 4, 8, 0, 0, p) == -2      # bf16 width not a multiple of 8
    assert lib.dp_sqnorms_dense(h, p + 2, p, 1, 1, 1, 8, 8, 0, 0, p) == -4  # bf16 pointer not 16-byte aligned
    assert lib.dp_sqnorms_dense(h, p, p, 0, 0, 5, 4, 4, 0, 0, p) == 0       # empty batch: no-op
    assert lib.dp_sqnorms_dense(None, p, p, 0, 1, 1, 4, 4, 0, 0, p) == -1
    assert lib.dp_clip_accumulate_dense(h, p, p, 0, 1, 1, 4, 4, 0.0, p, p, None) == -5
    assert lib.dp_clip_accumulate_dense(h, p, p, 0, 1, 1, 4, 4, float("nan"), p, p, None) == -5
    assert lib.dp_sqnorms_embedding(h, p, p, 0, 1, 1, 4, 0, 0, p) == -2
    assert lib.dp_sqnorms_embedding(h, p, p, 0, 1, 5000, 4, 10, 0, p) == -2   # T above the supported maximum
    kw = (p, p, p, p, 4, 0)
    assert lib.dp_noise_adamw(h, *kw, -1.0, 1.0, 0, 1, 8, 1e-3, 0.9, 0.999, 1e-11, 0.0, 0) == -5
    assert lib.dp_noise_adamw(h, *kw, 0.0, 1.0, 0, 0, 8, 1e-3, 0.9, 0.999, 1e-11, 0.0, 0) == -5   # step 0
    assert lib.dp_noise_adamw(h, *kw, 0.0, 1.0, 0, 1, 0, 1e-3, 0.9, 0.999, 1e-11, 0.0, 0) == -5   # batch 0
    assert lib.dp_noise_adamw(h, *kw, 0.0, 1.0, 0, 1, 8, 1e-3, 1.0, 0.999, 1e-11, 0.0, 0) == -5   # beta1 = 1
    assert lib.dp_noise_adamw(h, p, p, None, p, 4, 0, 0.0, 1.0, 0, 1, 8, 1e-3, 0.9, 0.999, 1e-11, 0.0, 0) == -1
    assert "beta" in pkg.dp_last_error(h) or pkg.dp_last_error(h)
    # tied table: (ctx, ids, dY, H, dL, dtype, B, T, M, d, V, ...)
    assert lib.dp_sqnorms_tied_embedding(h, p, p, p, p, 1, 1, 4, 2, 8, 12, p) == -2       # bf16: V not a multiple of 8
    assert lib.dp_sqnorms_tied_embedding(h, p, p, None, p, 0, 1, 4, 2, 8, 12, p) == -1    # M > 0 needs H
    assert lib.dp_sqnorms_tied_embedding(h, p, p, p, p, 0, 1, 4, 2, 8, 0, p) == -2        # V = 0
    assert lib.dp_sqnorms_tied_embedding(h, p, p, p, p, 0, 1, 4, -1, 8, 16, p) == -2      # negative M
    assert lib.dp_sqnorms_tied_embedding(h, p, p, p, p, 0, 0, 4, 2, 8, 16, p) == 0        # empty batch
    assert lib.dp_clip_accumulate_tied_embedding(h, p, p, p, p, 0, 1, 4, 2, 8, 16, -1.0, p, p) == -5
    assert lib.dp_clip_accumulate_tied_embedding(h, p, p, p, p, 1, 1, 4, 2, 8, 16, 1.0, p, p + 4) == -4  # bf16: sum_E alignment
    # pointer tables
    import ctypes
    tab = (ctypes.c_void_p * 2)(p, None)
    good = (ctypes.c_void_p * 2)(p, p)
    assert lib.dp_sqnorms_layernorm_batched(h, 2, tab, good, 0, 1, 1, 4, p) == -1
    assert lib.dp_sqnorms_layernorm_batched(h, 2, None, good, 0, 1, 1, 4, p) == -1
    assert lib.dp_sqnorms_layernorm_batched(h, -1, good, good, 0, 1, 1, 4, p) == -2
    assert lib.dp_sqnorms_layernorm_batched(h, 0, None, None, 0, 1, 1, 4, p) == 0
    assert lib.dp_clip_accumulate_layernorm_batched(h, 2, good, good, 0, 1, 1, 4, 1.0, p, good, tab) == -1
    assert lib.dp_clip_accumulate_layernorm_batched(h, 2, good, good, 0, 1, 1, 4, 0.0, p, good, good) == -5
    dp.sync()
    assert not host(x).any()


def test_small_workspace(dp):
    """A context with a 2 MiB workspace: the GEMM takes fewer row splits than it would like and still gives the
    oracle's sums; a call whose buffers cannot fit returns DP_ERR_WORKSPACE and leaves the context usable."""
    import paper_2108_01624_amd as pkg

    B, T, d_in, d_out, C = 64, 128, 512, 512, 1.0
    A, G = gen((B, T, d_in), 1.0, 900, "bf16"), gen((B, T, d_out), 0.1, 901, "bf16")
    sq = syn.synthetic_sqnorms(B, C, 902)
    W_ref, b_ref = orc.clip_accumulate_dense(A, G, orc.clip_factors(sq.astype(np.float64), C), True)
    big = torch.zeros(d_in, d_out, dtype=torch.float32, device=DEV)
    dp.clip_accumulate_dense(to_dev(A), to_dev(G), C, f32_dev(sq), big, None)
    dp.sync()
    with pkg.Context(workspace_bytes=2 << 20) as small:
        S = torch.zeros(d_in, d_out, dtype=torch.float32, device=DEV)
        Sb = torch.zeros(d_out, dtype=torch.float32, device=DEV)
        small.clip_accumulate_dense(to_dev(A), to_dev(G), C, f32_dev(sq), S, Sb)
        small.sync()
        assert_sums_close(host(S), W_ref, TOL_BF16, "sum_W, small workspace")
        assert_sums_close(host(S), host(big).astype(np.float64), 1e-5, "small against default workspace")
        assert_sums_close(host(Sb), b_ref, 1e-3, "sum_b, small workspace")
        # the embedding sums sort 8,192 tokens and keep two partial rows per 32-token chunk: 2 x 256 x 1024 floats
        V, d = 1000, 1024
        ids = to_dev(syn.zipf_ids(B, T, V, 1.1, 903))
        Ge = to_dev(gen((B, T, d), 0.1, 904, "bf16"))
        SE = torch.zeros(V, d, dtype=torch.float32, device=DEV)
        with pytest.raises(pkg.DpError) as e:
            small.clip_accumulate_embedding(ids, Ge, V, C, f32_dev(sq), SE)
        assert e.value.status == -7
        small.sync()
        assert not host(SE).any()
        n = torch.zeros(B, dtype=torch.float32, device=DEV)
        small.sqnorms_dense(to_dev(A), to_dev(G), True, pkg.DP_PATH_AUTO, n)   # still usable
        small.sync()
        n_ref = torch.zeros(B, dtype=torch.float32, device=DEV)
        dp.sqnorms_dense(to_dev(A), to_dev(G), True, pkg.DP_PATH_AUTO, n_ref)
        dp.sync()
        np.testing.assert_array_equal(host(n), host(n_ref))


def test_tiny_workspace_every_entry_point_works_or_reports(dp):
    """4 KiB of workspace: every call either needs none of it and gives the default context's result, or returns
    DP_ERR_WORKSPACE without touching its outputs."""
    import paper_2108_01624_amd as pkg

    B, T, d, V, C = 48, 128, 256, 300, 1.0
    A, G = to_dev(gen((B, T, d), 1.0, 910, "bf16")), to_dev(gen((B, T, d), 0.1, 911, "bf16"))
    A3, G3 = to_dev(gen((B, 50, 72), 1.0, 912, "bf16")), to_dev(gen((B, 50, 136), 0.1, 913, "bf16"))
    ids = to_dev(syn.zipf_ids(B, T, V, 1.1, 914))
    sq = f32_dev(syn.synthetic_sqnorms(B, C, 915))
    zeros = lambda *shape: torch.zeros(*shape, dtype=torch.float32, device=DEV)
    kw = dict(sigma=0.5, C=C, seed=3, step=1, batch_size=B, lr=1e-3, beta1=0.9, beta2=0.999, weight_decay=0.1)
    n_par = 100003
    S0 = syn.normal_f32((n_par,), 1.0, 916)

    def calls(ctx):
        """(name, outputs, thunk) for one context"""
        out = []
        for name, path in (("gram", pkg.DP_PATH_GRAM), ("materialise", pkg.DP_PATH_MATERIALISE)):
            n = zeros(B)
            out.append((f"sqnorms_dense {name}", [n], lambda n=n, path=path: ctx.sqnorms_dense(A, G, True, path, n)))
        n = zeros(B)
        out.append(("sqnorms_dense ragged", [n], lambda n=n: ctx.sqnorms_dense(A3, G3, True, pkg.DP_PATH_AUTO, n)))
        n = zeros(B)
        out.append(("sqnorms_layernorm", [n], lambda n=n: ctx.sqnorms_layernorm(A, G, n)))
        n = zeros(B)
        out.append(("sqnorms_embedding", [n], lambda n=n: ctx.sqnorms_embedding(ids, G, V, False, n)))
        W, b = zeros(d, d), zeros(d)
        out.append(("clip_accumulate_dense", [W, b], lambda W=W, b=b: ctx.clip_accumulate_dense(A, G, C, sq, W, b)))
        W, b = zeros(72, 136), zeros(136)
        out.append(("clip_accumulate_dense ragged", [W, b], lambda W=W, b=b: ctx.clip_accumulate_dense(A3, G3, C, sq, W, b)))
        g, be = zeros(d), zeros(d)
        out.append(("clip_accumulate_layernorm", [g, be], lambda g=g, be=be: ctx.clip_accumulate_layernorm(A, G, C, sq, g, be)))
        E = zeros(V, d)
        out.append(("clip_accumulate_embedding", [E], lambda E=E: ctx.clip_accumulate_embedding(ids, G, V, C, sq, E)))
        th, m, v, S, snr = zeros(n_par), zeros(n_par), zeros(n_par), f32_dev(S0), zeros(2)
        out.append(("noise_adamw_snr", [th, snr], lambda th=th, m=m, v=v, S=S, snr=snr: ctx.noise_adamw_snr(th, m, v, S, snr, **kw)))
        return out

    ref = calls(dp)
    for _, _, thunk in ref:
        thunk()
    dp.sync()
    reported = []
    with pkg.Context(workspace_bytes=4096) as tiny:
        for (name, outs, thunk), (_, ref_outs, _) in zip(calls(tiny), ref):
            try:
                thunk()
                tiny.sync()
            except pkg.DpError as e:
                assert e.status == -7, (name, e)
                tiny.sync()
                reported.append(name)
                for o in outs:
                    assert not host(o).any(), f"{name}: output touched although the call reported an error"
                continue
            for o, r in zip(outs, ref_outs):
                assert_sums_close(host(o), host(r).astype(np.float64), 1e-5, name)
    assert "clip_accumulate_embedding" in reported, reported   # the sort buffers of 6,144 tokens cannot fit in 4 KiB


def test_zero_and_empty_calls(dp):
    import paper_2108_01624_amd as pkg

    x = torch.ones(1003, dtype=torch.float32, device=DEV)
    dp.zero_f32(x[1:], n=1001)
    dp.sync()
    h = host(x)
    assert h[0] == 1 and h[-1] == 1 and not h[1:1002].any()
    n = torch.ones(4, dtype=torch.float32, device=DEV)
    e = torch.zeros(0, 16, 8, dtype=torch.bfloat16, device=DEV)
    lib = pkg.load_library()
    assert lib.dp_sqnorms_layernorm(dp.handle, n.data_ptr(), n.data_ptr(), 1, 0, 16, 8, n.data_ptr()) == 0
    assert lib.dp_clip_accumulate_layernorm(dp.handle, n.data_ptr(), n.data_ptr(), 1, 4, 0, 8, 1.0, n.data_ptr(), n.data_ptr(), n.data_ptr()) == 0
    dp.sync()
    assert host(n).tolist() == [1, 1, 1, 1]
    # kept LayerNorm gradients: no examples is a no-op; no tokens means zero gradients, written as such
    import ctypes
    d = 8
    keep = torch.full((4, 2, d), 3.0, dtype=torch.float32, device=DEV)
    x = torch.ones(4, 1, d, dtype=torch.float32, device=DEV)
    one = lambda t: (ctypes.c_void_p * 1)(t.data_ptr())
    assert lib.dp_sqnorms_layernorm_keep(dp.handle, 1, one(x), one(x), 0, 0, 1, d, n.data_ptr(), one(keep)) == 0
    dp.sync()
    assert float(host(keep).min()) == 3.0
    assert lib.dp_sqnorms_layernorm_keep(dp.handle, 1, one(x), one(x), 0, 4, 0, d, n.data_ptr(), one(keep)) == 0
    dp.sync()
    assert not host(keep).any() and host(n).tolist() == [1, 1, 1, 1]
    sg = torch.full((d,), 2.0, dtype=torch.float32, device=DEV)
    sb = torch.full((d,), 2.0, dtype=torch.float32, device=DEV)
    assert lib.dp_clip_accumulate_layernorm_kept(dp.handle, 1, one(keep), 0, d, 1.0, n.data_ptr(), one(sg), one(sb)) == 0
    assert lib.dp_clip_accumulate_layernorm_kept(dp.handle, 1, one(keep), 4, 6, 1.0, n.data_ptr(), one(sg), one(sb)) == -2  # d % 4
    dp.sync()
    assert host(sg).tolist() == [2.0] * d and host(sb).tolist() == [2.0] * d


@pytest.mark.parametrize("dtype,B,T,d,V", [("bf16", 9, 128, 64, 512), ("bf16", 3, 7, 8, 16), ("f32", 5, 33, 20, 40),
                                           ("bf16", 70, 16, 256, 16)])
def test_clip_accumulate_positions(dp, dtype, B, T, d, V):
    """Position embedding without the sort: against the oracle's scatter with ids 0..T-1 and against the general path."""
    C = 1.0
    G = gen((B, T, d), 0.1, 700, dtype)
    ids = syn.position_ids(B, T)
    sq = syn.synthetic_sqnorms(B, C, 701)
    c = orc.clip_factors(sq.astype(np.float64), C)
    ref = orc.clip_accumulate_embedding(ids, G, c, V)
    init = syn.normal_f32((V, d), float(np.abs(ref).mean()), 702)
    S_fast, S_gen = f32_dev(init), f32_dev(init)
    dp.clip_accumulate_positions(to_dev(G), C, f32_dev(sq), S_fast)
    dp.clip_accumulate_embedding(to_dev(ids), to_dev(G), V, C, f32_dev(sq), S_gen)
    dp.sync()
    tol = 1e-5 if dtype == "f32" else 1e-4
    assert_sums_close(host(S_fast) - init.astype(np.float64), ref, tol, "positions")
    np.testing.assert_array_equal(host(S_fast)[T:], init[T:])          # rows from T on are untouched
    np.testing.assert_allclose(host(S_fast), host(S_gen), rtol=1e-4, atol=1e-6 * np.abs(ref).max())


# ------------------------------------------------------------------------------------------------
# a table used as lookup and as output projection (tied weights)
# ------------------------------------------------------------------------------------------------
def _tied_case(dtype, B, T, M, d, V, seed):
    ids = syn.zipf_ids(B, T, V, 1.1, seed)
    dY = gen((B, T, d), 0.3, seed + 1, dtype)
    H = gen((B, M, d), 1.0, seed + 2, dtype)
    dLf = syn.normal_f32((B, M, V), 0.02, seed + 3)
    labels = syn.zipf_ids(B, max(M, 1), V, 1.1, seed + 4)
    for i in range(B):
        for m in range(M):
            dLf[i, m, labels[i, m]] -= 0.5               # the label's column, as in a cross-entropy gradient
            if m < min(M, T) and i % 2 == 0:
                dLf[i, m, ids[i, m]] -= 0.25             # predicted tokens that also occur in the input: a large cross term
    if M > 1:
        dLf[B // 2, M - 1] = 0.0                         # an unused prediction slot
    dL = syn.f32_to_bf16_bits(dLf) if dtype == "bf16" else dLf
    return ids, dY, H, dL


@pytest.mark.parametrize("dtype,B,T,M,d,V", [("bf16", 6, 128, 20, 128, 1024), ("bf16", 3, 40, 5, 72, 200), ("bf16", 2, 160, 80, 64, 512),
                                             ("bf16", 4, 33, 33, 8, 64), ("f32", 5, 19, 7, 20, 50), ("f32", 2, 70, 3, 130, 33),
                                             ("bf16", 3, 16, 0, 64, 64), ("bf16", 16, 24, 20, 256, 520),
                                             # enough rows that the projection's GEMM splits them: partial sums next to
                                             # the pre-scaled H that the caller holds in the same workspace
                                             ("bf16", 64, 24, 20, 256, 520)])
def test_tied_embedding_norms_and_sums(dp, dtype, B, T, M, d, V):
    ids, dY, H, dL = _tied_case(dtype, B, T, M, d, V, 800)
    n0 = np.linspace(0.5, 1.5, B).astype(np.float32)     # the entry point adds to what is there
    n = f32_dev(n0)
    args = (to_dev(ids), to_dev(dY), to_dev(H), to_dev(dL))
    dp.sqnorms_tied_embedding(*args, n)
    dp.sync()
    ref = orc.sqnorms_tied_embedding(ids, dY, H, dL)
    # bf16 products are exact in fp32 on both sides; what is left is fp32 summation order
    tol = 2e-5 if dtype == "f32" else 1e-4
    assert_norms_close(host(n).astype(np.float64) - n0, ref, tol, "tied norms")
    if M and T:
        parts = orc.sqnorms_embedding(ids, dY, V) + orc.sqnorms_dense(dL, H, False)
        assert np.abs(ref - parts).max() > 20 * tol * ref.max()   # dropping the cross term would be far outside the bound
    C = float(np.sqrt(np.median(ref)))                   # about half of the examples clipped
    sq = ref.astype(np.float32)
    c = orc.clip_factors(sq.astype(np.float64), C)
    S_ref = orc.clip_accumulate_tied_embedding(ids, dY, H, dL, c)
    init = syn.normal_f32((V, d), float(np.abs(S_ref).mean()), 801)
    S = f32_dev(init)
    dp.clip_accumulate_tied_embedding(*args, C, f32_dev(sq), S)
    dp.sync()
    assert_sums_close(host(S).astype(np.float64) - init, S_ref, 1e-5 if dtype == "f32" else TOL_BF16, "tied sum")


def test_tied_embedding_out_of_range_id_is_reported(dp):
    import paper_2108_01624_amd as pkg

    ids, dY, H, dL = _tied_case("bf16", 2, 8, 3, 8, 16, 810)
    ids[1, 2] = 16
    n = torch.zeros(2, dtype=torch.float32, device=DEV)
    dp.sqnorms_tied_embedding(to_dev(ids), to_dev(dY), to_dev(H), to_dev(dL), n)
    with pytest.raises(pkg.DpError) as e:
        dp.sync()
    assert e.value.status == -6
    dp.sync()


# ------------------------------------------------------------------------------------------------
# several same-shaped dense layers in one call
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("n,B,T,d_in,d_out", [(3, 8, 128, 256, 384), (18, 2, 32, 256, 256), (5, 16, 128, 512, 256),
                                              (2, 3, 50, 512, 264), (3, 4, 64, 72, 136),
                                              # 9 and 36 tiles per layer: workgroup counts that are no multiple of 8
                                              # (the balanced XCD mapping, with and without the rectangle walk)
                                              (5, 12, 128, 768, 768), (3, 4, 128, 768, 3072),
                                              # widths that end inside a 256-column tile, odd layer counts, T = one and three stages of 64 rows
                                              (7, 6, 64, 264, 520), (2, 20, 192, 1000, 256)])
def test_clip_accumulate_dense_batched(dp, n, B, T, d_in, d_out):
    C = 1.0
    sq = syn.synthetic_sqnorms(B, C, 300)
    c = orc.clip_factors(sq.astype(np.float64), C)
    As = [gen((B, T, d_in), 1.0, 310 + l, "bf16") for l in range(n)]
    Gs = [gen((B, T, d_out), 0.1, 340 + l, "bf16") for l in range(n)]
    SW = [torch.full((d_in, d_out), 0.25, dtype=torch.float32, device=DEV) for _ in range(n)]
    Sb = [torch.full((d_out,), -0.5, dtype=torch.float32, device=DEV) if l != 1 else None for l in range(n)]
    dp.clip_accumulate_dense_batched([to_dev(a) for a in As], [to_dev(g) for g in Gs], C, f32_dev(sq), SW, Sb)
    dp.sync()
    for l in range(n):
        W_ref, b_ref = orc.clip_accumulate_dense(As[l], Gs[l], c, True)
        rel = assert_sums_close(host(SW[l]).astype(np.float64) - 0.25, W_ref, TOL_BF16, f"layer {l} sum_W")
        assert rel < 5e-3
        if Sb[l] is not None:
            assert_sums_close(host(Sb[l]).astype(np.float64) + 0.5, b_ref, 1e-3, f"layer {l} sum_b")


def test_batched_equals_single_layer_calls(dp):
    """The direct-to-LDS path keeps exact bf16 products: one layer alone and inside a batch agree closely."""
    n, B, T, d_in, d_out, C = 4, 32, 128, 256, 256, 1.0
    sq = f32_dev(syn.synthetic_sqnorms(B, C, 301))
    As = [to_dev(gen((B, T, d_in), 1.0, 400 + l, "bf16")) for l in range(n)]
    Gs = [to_dev(gen((B, T, d_out), 0.1, 420 + l, "bf16")) for l in range(n)]
    one = [torch.zeros(d_in, d_out, dtype=torch.float32, device=DEV) for _ in range(n)]
    bat = [torch.zeros(d_in, d_out, dtype=torch.float32, device=DEV) for _ in range(n)]
    for l in range(n):
        dp.clip_accumulate_dense(As[l], Gs[l], C, sq, one[l], None)
    dp.clip_accumulate_dense_batched(As, Gs, C, sq, bat, None)
    dp.sync()
    for l in range(n):
        assert_sums_close(host(bat[l]), host(one[l]).astype(np.float64), 1e-5, f"layer {l}")


@pytest.mark.parametrize("n,B,T,d_in,d_out,has_bias", [(3, 5, 128, 256, 384, True), (18, 3, 96, 64, 128, False),
                                                        (2, 4, 100, 72, 136, True), (2, 2, 300, 128, 128, True),
                                                        (1, 6, 128, 128, 64, True)])
def test_sqnorms_dense_batched(dp, n, B, T, d_in, d_out, has_bias):
    """n same-shaped layers in one call: fast-path shapes (shared launches, more than 16 layers), ragged shapes and
    several Gram blocks (per-layer fallback); the norms of all layers add up, on top of what sqnorms held."""
    import paper_2108_01624_amd as pkg

    As = [gen((B, T, d_in), 1.0, 500 + l, "bf16") for l in range(n)]
    Gs = [gen((B, T, d_out), 0.1, 540 + l, "bf16") for l in range(n)]
    ref = sum(orc.sqnorms_dense(a, g, has_bias) for a, g in zip(As, Gs))
    A_d, G_d = [to_dev(a) for a in As], [to_dev(g) for g in Gs]
    for path in (pkg.DP_PATH_AUTO, pkg.DP_PATH_GRAM, pkg.DP_PATH_MATERIALISE):
        out = torch.full((B,), 3.0, dtype=torch.float32, device=DEV)
        dp.sqnorms_dense_batched(A_d, G_d, has_bias, path, out)
        dp.sync()
        assert_norms_close(host(out).astype(np.float64) - 3.0, ref, 1e-4, f"path {path}")
    # bit-reproducible, and equal to layer-by-layer calls up to the order of the fp32 additions
    one = torch.zeros(B, dtype=torch.float32, device=DEV)
    two = torch.zeros(B, dtype=torch.float32, device=DEV)
    seq = torch.zeros(B, dtype=torch.float32, device=DEV)
    dp.sqnorms_dense_batched(A_d, G_d, has_bias, pkg.DP_PATH_GRAM, one)
    dp.sqnorms_dense_batched(A_d, G_d, has_bias, pkg.DP_PATH_GRAM, two)
    for a, g in zip(A_d, G_d):
        dp.sqnorms_dense(a, g, has_bias, pkg.DP_PATH_GRAM, seq)
    dp.sync()
    np.testing.assert_array_equal(host(one), host(two))
    np.testing.assert_allclose(host(one), host(seq), rtol=1e-6)


@pytest.mark.parametrize("ng,n_out,B,T,d_in,d_out,has_bias", [(2, 3, 5, 128, 256, 128, True), (1, 2, 3, 64, 64, 192, False),
                                                               (18, 3, 2, 32, 64, 64, True), (2, 3, 2, 300, 128, 128, True),
                                                               (1, 3, 4, 100, 72, 136, True)])
def test_sqnorms_dense_shared_input(dp, ng, n_out, B, T, d_in, d_out, has_bias):
    """Groups of layers reading one input (query / key / value): the norms are those of ng * n_out separate layers
    (the oracle knows nothing of the sharing); fast-path shapes, more than 16 groups, and per-layer fallbacks."""
    As = [gen((B, T, d_in), 1.0, 600 + g, "bf16") for g in range(ng)]
    Gs = [[gen((B, T, d_out), 0.1, 640 + 4 * g + j, "bf16") for j in range(n_out)] for g in range(ng)]
    ref = sum(orc.sqnorms_dense(As[g], Gs[g][j], has_bias) for g in range(ng) for j in range(n_out))
    A_d = [to_dev(a) for a in As]
    G_d = [[to_dev(x) for x in gs] for gs in Gs]
    out = torch.full((B,), 2.0, dtype=torch.float32, device=DEV)
    dp.sqnorms_dense_shared(A_d, G_d, has_bias, out)
    dp.sync()
    assert_norms_close(host(out).astype(np.float64) - 2.0, ref, 1e-4, "shared input")


def test_step_runner_uses_shared_inputs(dp):
    """A manifest whose q/k/v layers are handed the same input tensor gives the norms of the separate-layer definition."""
    import paper_2108_01624_amd as pkg

    man = syn.bert_manifest(1, 128, 256)
    B, T = 4, 128
    layers = syn.device_layer_inputs(man, B, T, dtype="bf16", act_std=1.0, grad_std=1e-2, data_seed=77, device=DEV)
    q, k, v = [l for l in layers if l["kind"] == "dense"][:3]
    k["A"] = q["A"]
    v["A"] = q["A"]
    run = pkg.StepRunner(dp, man, B, device=DEV)
    n = run.pass1(layers)
    dp.sync()
    n_ref = orc.microbatch_sqnorms(syn.host_layer_slice(layers, range(B)))
    assert_norms_close(host(n), n_ref, 1e-4, "norms with shared q/k/v input")
    n_sep = host(run.pass1(layers, batch_dense=False)).copy()
    dp.sync()
    np.testing.assert_allclose(host(n), n_sep, rtol=1e-5)


# ------------------------------------------------------------------------------------------------
# Philox against an independent library (needs the HIP runtime, hence a GPU-box test)
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("seed,offset,n", [(0, 0, 64), (0x0123456789ABCDEF, 0, 4096), (2 ** 64 - 1, 4096, 1000),
                                           (42, 7, 33), (1234, 4 * (2 ** 32) - 8, 64)])
def test_philox_matches_rocrand_host_generator(dp, seed, offset, n):
    """rocRAND's host-side Philox4x32-10 generator (seed -> key, stream offset -> counter, four words per
    counter) is an implementation of the same published rounds by other hands: the oracle and the HIP kernel
    must give its words bit for bit (step = 0 leaves the upper counter words zero, as rocRAND has them)."""
    import ctypes

    try:
        lib = ctypes.CDLL("/opt/rocm/lib/librocrand.so")
    except OSError:
        pytest.skip("librocrand.so not available")
    gen = ctypes.c_void_p()
    if lib.rocrand_create_generator_host_blocking(ctypes.byref(gen), 404) != 0:  # ROCRAND_RNG_PSEUDO_PHILOX4_32_10
        pytest.skip("rocRAND host generator cannot be created here")
    try:
        assert lib.rocrand_set_seed(gen, ctypes.c_ulonglong(seed)) == 0
        assert lib.rocrand_set_offset(gen, ctypes.c_ulonglong(offset)) == 0
        ref = np.zeros(n, dtype=np.uint32)
        assert lib.rocrand_generate(gen, ref.ctypes.data_as(ctypes.c_void_p), ctypes.c_size_t(n)) == 0
    finally:
        lib.rocrand_destroy_generator(gen)
    np.testing.assert_array_equal(orc.philox_u32(n, offset, seed, 0), ref)
    out = torch.zeros(n, dtype=torch.int32, device=DEV)
    dp.philox_u32(out, offset, seed, 0)
    dp.sync()
    np.testing.assert_array_equal(host(out).view(np.uint32), ref)
