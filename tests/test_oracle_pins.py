"""Pins of the CPU oracle to things other than itself: brute-force autograd, closed forms,
invariants, library routines (flat GEMM, bincount, torch.optim.AdamW), statistics of the noise."""
import math
import os

import numpy as np
import pytest
import torch

import dp_synth as syn
from oracle import dp_oracle as orc



# ----------------------------------------------------------------------------------------------
# brute-force autograd on a tiny BERT-like model
# ----------------------------------------------------------------------------------------------
def _tiny_model(B=5, T=7, d=6, dff=10, V=11, seed=0):
    g = torch.Generator().manual_seed(seed)
    rn = lambda *s: torch.randn(*s, generator=g, dtype=torch.float64)
    P = dict(E_tok=rn(V, d), E_pos=rn(T + 2, d), ln0_g=1 + 0.1 * rn(d), ln0_b=0.1 * rn(d),
             W1=rn(d, dff) / math.sqrt(d), b1=0.1 * rn(dff), W2=rn(dff, d) / math.sqrt(dff), b2=0.1 * rn(d),
             ln1_g=1 + 0.1 * rn(d), ln1_b=0.1 * rn(d))
    for p in P.values():
        p.requires_grad_(True)
    ids = torch.randint(0, V, (B, T), generator=g)
    ids[:, 3] = ids[:, 1]  # force repeated ids inside every example
    ids[0, :] = 4          # one example with a single id
    tgt = rn(B, T, d)
    return P, ids, tgt


def _forward(P, ids, tgt, keep=None):
    T = ids.shape[-1]
    e = P["E_tok"][ids] + P["E_pos"][torch.arange(T)]
    xh0 = (e - e.mean(-1, keepdim=True)) / torch.sqrt(e.var(-1, unbiased=False, keepdim=True) + 1e-5)
    h0 = xh0 * P["ln0_g"] + P["ln0_b"]
    y1 = h0 @ P["W1"] + P["b1"]
    a1 = torch.nn.functional.gelu(y1)
    y2 = a1 @ P["W2"] + P["b2"]
    r = y2 + h0
    xh1 = (r - r.mean(-1, keepdim=True)) / torch.sqrt(r.var(-1, unbiased=False, keepdim=True) + 1e-5)
    out = xh1 * P["ln1_g"] + P["ln1_b"]
    loss_per_example = ((out - tgt) ** 2).sum(dim=(-1, -2))
    if keep is not None:
        for k, t in dict(e=e, xh0=xh0, h0=h0, y1=y1, a1=a1, y2=y2, xh1=xh1, out=out).items():
            t.retain_grad()
            keep[k] = t
    return loss_per_example


def _capture_layers(P, ids, tgt):
    """Batched forward/backward of sum_i loss_i: since loss_i only depends on example i, the gradient
    w.r.t. each layer output is, row by row, the gradient of that example's own loss."""
    keep = {}
    _forward(P, ids, tgt, keep).sum().backward()
    for p in P.values():
        p.grad = None
    npy = lambda t: t.detach().numpy().copy()
    V, Tp = P["E_tok"].shape[0], P["E_pos"].shape[0]
    B, T = ids.shape
    layers = [
        dict(kind="embedding", ids=ids.numpy().astype(np.int32), G=npy(keep["e"].grad), V=V),
        dict(kind="embedding", ids=syn.position_ids(B, T), G=npy(keep["e"].grad), V=Tp),
        # h0 feeds dense1 AND the residual: its retained grad is the total gradient of the LayerNorm output
        dict(kind="layernorm", X=npy(keep["xh0"]), G=npy(keep["h0"].grad)),
        dict(kind="dense", A=npy(keep["h0"]), G=npy(keep["y1"].grad), has_bias=True),
        dict(kind="dense", A=npy(keep["a1"]), G=npy(keep["y2"].grad), has_bias=True),
        dict(kind="layernorm", X=npy(keep["xh1"]), G=npy(keep["out"].grad)),
    ]
    return layers


PARAM_ORDER = [["E_tok"], ["E_pos"], ["ln0_g", "ln0_b"], ["W1", "b1"], ["W2", "b2"], ["ln1_g", "ln1_b"]]


def _per_example_autograd(P, ids, tgt):
    B = ids.shape[0]
    grads = []
    for i in range(B):
        for p in P.values():
            p.grad = None
        _forward(P, ids[i:i + 1], tgt[i:i + 1]).sum().backward()
        grads.append({k: (p.grad.detach().numpy().copy() if p.grad is not None else np.zeros(tuple(p.shape)))
                      for k, p in P.items()})
    return grads


@pytest.mark.parametrize("Cclip", [0.5, 3.0, 1e9])
def test_autograd_bruteforce_tiny_bert(Cclip):
    P, ids, tgt = _tiny_model()
    layers = _capture_layers(P, ids, tgt)
    grads = _per_example_autograd(P, ids, tgt)
    B = ids.shape[0]
    n_true = np.array([sum(float((g ** 2).sum()) for g in grads[i].values()) for i in range(B)])
    c_true = np.minimum(1.0, Cclip / np.sqrt(n_true))
    sums, n, c = orc.microbatch_clip_sum(layers, Cclip)
    np.testing.assert_allclose(n, n_true, rtol=1e-10)
    np.testing.assert_allclose(orc.microbatch_sqnorms(layers), n_true, rtol=1e-10)
    np.testing.assert_allclose(c, c_true, rtol=1e-10)
    if Cclip == 0.5:
        assert (c < 1).any()
    for s, names in zip(sums, PARAM_ORDER):
        for arr, nm in zip(s, names):
            ref = sum(c_true[i] * grads[i][nm] for i in range(B))
            np.testing.assert_allclose(arr, ref, rtol=1e-9, atol=1e-12, err_msg=nm)
    # per-layer entry points agree with the autograd per-example gradients too
    n_dense = orc.sqnorms_dense(layers[3]["A"], layers[3]["G"], True)
    np.testing.assert_allclose(n_dense, [float((grads[i]["W1"] ** 2).sum() + (grads[i]["b1"] ** 2).sum()) for i in range(B)],
                               rtol=1e-10)
    n_nobias = orc.sqnorms_dense(layers[3]["A"], layers[3]["G"], False)
    np.testing.assert_allclose(n_nobias, [float((grads[i]["W1"] ** 2).sum()) for i in range(B)], rtol=1e-10)
    n_ln = orc.sqnorms_layernorm(layers[5]["X"], layers[5]["G"])
    np.testing.assert_allclose(n_ln, [float((grads[i]["ln1_g"] ** 2).sum() + (grads[i]["ln1_b"] ** 2).sum()) for i in range(B)],
                               rtol=1e-10)
    n_emb = orc.sqnorms_embedding(layers[0]["ids"], layers[0]["G"], layers[0]["V"])
    np.testing.assert_allclose(n_emb, [float((grads[i]["E_tok"] ** 2).sum()) for i in range(B)], rtol=1e-10)
    n_pos = orc.sqnorms_embedding(layers[1]["ids"], layers[1]["G"], layers[1]["V"])
    np.testing.assert_allclose(n_pos, [float((grads[i]["E_pos"] ** 2).sum()) for i in range(B)], rtol=1e-10)
    S_E = orc.clip_accumulate_embedding(layers[0]["ids"], layers[0]["G"], c_true, layers[0]["V"])
    np.testing.assert_allclose(S_E, sum(c_true[i] * grads[i]["E_tok"] for i in range(B)), rtol=1e-9, atol=1e-12)
    S_W, S_b = orc.clip_accumulate_dense(layers[4]["A"], layers[4]["G"], c_true, True)
    np.testing.assert_allclose(S_W, sum(c_true[i] * grads[i]["W2"] for i in range(B)), rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(S_b, sum(c_true[i] * grads[i]["b2"] for i in range(B)), rtol=1e-9, atol=1e-12)
    S_g, S_bb = orc.clip_accumulate_layernorm(layers[2]["X"], layers[2]["G"], c_true)
    np.testing.assert_allclose(S_g, sum(c_true[i] * grads[i]["ln0_g"] for i in range(B)), rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(S_bb, sum(c_true[i] * grads[i]["ln0_b"] for i in range(B)), rtol=1e-9, atol=1e-12)


# ----------------------------------------------------------------------------------------------
# closed forms for the dense norm
# ----------------------------------------------------------------------------------------------
def test_dense_T1_closed_form():
    A = syn.normal_f32((6, 1, 9), 1.0, 1)
    G = syn.normal_f32((6, 1, 5), 0.3, 2)
    n = orc.sqnorms_dense(A, G, False)
    a2 = (A.astype(np.float64) ** 2).sum(axis=(1, 2))
    g2 = (G.astype(np.float64) ** 2).sum(axis=(1, 2))
    np.testing.assert_allclose(n, a2 * g2, rtol=1e-12)
    np.testing.assert_allclose(orc.sqnorms_dense(A, G, True), a2 * g2 + g2, rtol=1e-12)


def test_dense_rank_one_G():
    """G_i = w u^T  =>  A^T G = (A^T w) u^T  and  ||.||_F^2 = ||A^T w||^2 ||u||^2."""
    rng = np.random.default_rng(3)
    A = rng.standard_normal((3, 8, 5))
    w = rng.standard_normal((3, 8))
    u = rng.standard_normal((3, 4))
    G = w[:, :, None] * u[:, None, :]
    ref = [np.sum((A[i].T @ w[i]) ** 2) * np.sum(u[i] ** 2) for i in range(3)]
    np.testing.assert_allclose(orc.sqnorms_dense(A, G, False), ref, rtol=1e-12)


def test_dense_gram_identity_bruteforce():
    """||A^T G||_F^2 = sum_{t,s} (a_t.a_s)(g_t.g_s), evaluated with scalar loops."""
    rng = np.random.default_rng(4)
    A = rng.standard_normal((2, 5, 3))
    G = rng.standard_normal((2, 5, 4))
    for i in range(2):
        tot = 0.0
        bias = 0.0
        for t in range(5):
            for s in range(5):
                aa = sum(A[i, t, p] * A[i, s, p] for p in range(3))
                gg = sum(G[i, t, q] * G[i, s, q] for q in range(4))
                tot += aa * gg
                bias += gg
        assert math.isclose(orc.sqnorms_dense(A, G, False)[i], tot, rel_tol=1e-12)
        assert math.isclose(orc.sqnorms_dense(A, G, True)[i], tot + bias, rel_tol=1e-12)


def test_dense_orientation():
    """S_W is [d_in, d_out]: entry (p, q) pairs input feature p with output feature q."""
    A = np.zeros((1, 2, 3))
    G = np.zeros((1, 2, 4))
    A[0, 0, 2] = 2.0
    G[0, 0, 1] = 3.0
    S_W, _ = orc.clip_accumulate_dense(A, G, np.ones(1), False)
    assert S_W.shape == (3, 4)
    assert S_W[2, 1] == 6.0 and np.count_nonzero(S_W) == 1
    # square layer (the attention projections): the shape cannot reveal a transposed product, the entry does
    A = np.zeros((1, 2, 4))
    A[0, 1, 3] = 5.0
    G[0, 1, 0] = 7.0
    S_W, _ = orc.clip_accumulate_dense(A, G, np.ones(1), False)
    assert S_W[3, 0] == 35.0 and np.count_nonzero(S_W) == 1
    gW, _ = orc.dense_example_grads(A[0], G[0])
    assert gW[3, 0] == 35.0 and gW[0, 3] == 0.0


# ----------------------------------------------------------------------------------------------
# clipping: invariant, no-op, both branches
# ----------------------------------------------------------------------------------------------
def _c1_like(B=8, T=16, d_in=24, d_out=16, seed=10, scale=None):
    A = syn.normal_f32((B, T, d_in), 1.0, seed)
    G = syn.normal_f32((B, T, d_out), 0.1, seed + 1)
    if scale is not None:
        G = (G * scale[:, None, None]).astype(np.float32)
    return A, G


def test_clip_invariant_and_all_clipped():
    A, G = _c1_like()
    C = 1.0
    n = orc.sqnorms_dense(A, G, True)
    c = orc.clip_factors(n, C)
    assert (c < 1).all()  # with these distributions every example is clipped
    for i in range(A.shape[0]):
        gW, gb = orc.dense_example_grads(A[i], G[i])
        clipped = math.sqrt(np.sum((c[i] * gW) ** 2) + np.sum((c[i] * gb) ** 2))
        assert clipped <= C * (1 + 1e-12)
        assert math.isclose(clipped, C, rel_tol=1e-12)


def test_clip_noop_equals_flat_gemm():
    A, G = _c1_like()
    n = orc.sqnorms_dense(A, G, True)
    C = 10.0 * math.sqrt(n.max())
    c = orc.clip_factors(n, C)
    assert (c == 1.0).all()
    S_W, S_b = orc.clip_accumulate_dense(A, G, c, True)
    Af = torch.from_numpy(A.reshape(-1, A.shape[2]).astype(np.float64))
    Gf = torch.from_numpy(G.reshape(-1, G.shape[2]).astype(np.float64))
    np.testing.assert_allclose(S_W, torch.matmul(Af.T, Gf).numpy(), rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(S_b, Gf.sum(0).numpy(), rtol=1e-11, atol=1e-13)


def test_sampled_entries_equal_full_sum():
    A, G = _c1_like(B=5, T=7, d_in=6, d_out=4, seed=40)
    c = np.linspace(0.2, 1.0, 5)
    S_W, _ = orc.clip_accumulate_dense(A, G, c, False)
    ps, qs = np.array([0, 5, 2, 3]), np.array([3, 0, 2, 1])
    got = orc.clip_accumulate_dense_entries(A[:, :, ps], G[:, :, qs], c)
    np.testing.assert_allclose(got, S_W[ps, qs], rtol=1e-12)


def test_clip_mixed_branches():
    B = 16
    scale = syn.example_scales(B, 1e-4, 1.0, 5)
    A, G = _c1_like(B=B, scale=scale)
    n = orc.sqnorms_dense(A, G, False)
    C = float(np.sqrt(np.median(n)))
    c = orc.clip_factors(n, C)
    assert (c == 1.0).any() and (c < 1.0).any()
    assert np.all(c * np.sqrt(n) <= C * (1 + 1e-12))
    np.testing.assert_allclose(c[c < 1] * np.sqrt(n[c < 1]), C, rtol=1e-12)


def test_clip_zero_gradient_gets_factor_one():
    assert orc.clip_factors(np.array([0.0, 4.0]), 1.0).tolist() == [1.0, 0.5]


# ----------------------------------------------------------------------------------------------
# embeddings
# ----------------------------------------------------------------------------------------------
def test_embedding_counts_and_index_add():
    B, T, V, d = 6, 20, 13, 4
    ids = syn.zipf_ids(B, T, V, 1.1, 7)
    ones = np.ones((B, T, d), dtype=np.float32)
    S = orc.clip_accumulate_embedding(ids, ones, np.ones(B), V)
    cnt = np.bincount(ids.reshape(-1), minlength=V)
    np.testing.assert_array_equal(S[:, 0], cnt.astype(np.float64))
    assert set(np.nonzero(S[:, 0])[0]) == set(np.unique(ids))
    # per-example norm with all-ones gradients: sum_v count_v^2 * d
    n = orc.sqnorms_embedding(ids, ones, V)
    ref = [d * float((np.bincount(r, minlength=V) ** 2).sum()) for r in ids]
    np.testing.assert_allclose(n, ref, rtol=0)
    # general gradients, weights c: torch.index_add_
    G = syn.normal_f32((B, T, d), 1.0, 8)
    c = np.linspace(0.1, 1.0, B)
    S = orc.clip_accumulate_embedding(ids, G, c, V)
    ref = torch.zeros(V, d, dtype=torch.float64)
    ref.index_add_(0, torch.from_numpy(ids.reshape(-1).astype(np.int64)),
                   torch.from_numpy((G.astype(np.float64) * c[:, None, None]).reshape(-1, d)))
    np.testing.assert_allclose(S, ref.numpy(), rtol=1e-12, atol=1e-14)


def test_position_embedding_closed_form():
    B, T, V, d = 4, 9, 16, 5
    G = syn.normal_f32((B, T, d), 1.0, 9)
    ids = syn.position_ids(B, T)
    n = orc.sqnorms_embedding(ids, G, V)
    np.testing.assert_allclose(n, (G.astype(np.float64) ** 2).sum(axis=(1, 2)), rtol=1e-12)
    S = orc.clip_accumulate_embedding(ids, G, np.ones(B), V)
    assert np.all(S[T:] == 0.0)
    np.testing.assert_allclose(S[:T], G.astype(np.float64).sum(axis=0), rtol=1e-12)


def test_embedding_rejects_out_of_range():
    with pytest.raises(IndexError):
        orc.sqnorms_embedding(np.array([[0, 5]], dtype=np.int32), np.ones((1, 2, 3), np.float32), 5)


# ----------------------------------------------------------------------------------------------
# a table used as lookup AND as output projection (tied weights)
# ----------------------------------------------------------------------------------------------


def _tied_model(B=4, T=6, M=3, d=5, V=9, seed=3):
    g = torch.Generator().manual_seed(seed)
    rn = lambda *s: torch.randn(*s, generator=g, dtype=torch.float64)
    P = dict(E=rn(V, d), W=rn(d, d) / math.sqrt(d))
    for p in P.values():
        p.requires_grad_(True)
    ids = torch.randint(0, V, (B, T), generator=g)
    ids[:, 2] = ids[:, 0]                               # repeated ids inside every example
    mpos = torch.stack([torch.randperm(T, generator=g)[:M] for _ in range(B)])
    labels = torch.randint(0, V, (B, M), generator=g)
    labels[1, 0] = ids[1, 0]                            # a label that is also one of the example's input ids
    w = torch.ones(B, M, dtype=torch.float64)
    w[2, M - 1] = 0.0                                   # a padded prediction slot
    return P, ids, mpos, labels, w


def _tied_forward(P, ids, mpos, labels, w, keep=None):
    B = ids.shape[0]
    x = P["E"][ids]                                     # lookup
    xw = x @ P["W"]
    hm = torch.tanh(xw)[torch.arange(B)[:, None], mpos]  # the M selected positions
    logits = hm @ P["E"].T                              # output projection with the SAME table
    if keep is not None:
        for k, t in dict(x=x, xw=xw, hm=hm, logits=logits).items():
            t.retain_grad()
            keep[k] = t
    ce = torch.nn.functional.cross_entropy(logits.reshape(-1, logits.shape[-1]), labels.reshape(-1), reduction="none")
    return (ce.reshape(B, -1) * w).sum(dim=1)


@pytest.mark.parametrize("Cclip", [0.3, 1e9])
def test_tied_embedding_against_autograd(Cclip):
    P, ids, mpos, labels, w = _tied_model()
    B = ids.shape[0]
    keep = {}
    _tied_forward(P, ids, mpos, labels, w, keep).sum().backward()
    npy = lambda t: t.detach().numpy().copy()
    ids_n = ids.numpy().astype(np.int32)
    dY, H, dL = npy(keep["x"].grad), npy(keep["hm"]), npy(keep["logits"].grad)
    assert np.all(dL[2, -1] == 0.0)                     # the padded slot has no gradient
    layers = [dict(kind="tied_embedding", ids=ids_n, G=dY, H=H, dL=dL, V=P["E"].shape[0]),
              dict(kind="dense", A=npy(keep["x"]), G=npy(keep["xw"].grad), has_bias=False)]
    grads = []
    for i in range(B):
        for p in P.values():
            p.grad = None
        _tied_forward(P, ids[i:i + 1], mpos[i:i + 1], labels[i:i + 1], w[i:i + 1]).sum().backward()
        grads.append({k: npy(p.grad) for k, p in P.items()})
    for i in range(B):
        g = orc.tied_embedding_example_grad(ids_n[i], dY[i], H[i], dL[i])
        np.testing.assert_allclose(g, grads[i]["E"], rtol=1e-10, atol=1e-13)
    n_E = np.array([float((grads[i]["E"] ** 2).sum()) for i in range(B)])
    np.testing.assert_allclose(orc.sqnorms_tied_embedding(ids_n, dY, H, dL), n_E, rtol=1e-10)
    n_true = n_E + np.array([float((grads[i]["W"] ** 2).sum()) for i in range(B)])
    c_true = np.minimum(1.0, Cclip / np.sqrt(n_true))
    sums, n, c = orc.microbatch_clip_sum(layers, Cclip)
    np.testing.assert_allclose(n, n_true, rtol=1e-10)
    np.testing.assert_allclose(orc.microbatch_sqnorms(layers), n_true, rtol=1e-10)
    np.testing.assert_allclose(c, c_true, rtol=1e-10)
    np.testing.assert_allclose(sums[0][0], sum(c_true[i] * grads[i]["E"] for i in range(B)), rtol=1e-9, atol=1e-13)
    np.testing.assert_allclose(sums[1][0], sum(c_true[i] * grads[i]["W"] for i in range(B)), rtol=1e-9, atol=1e-13)
    np.testing.assert_allclose(orc.clip_accumulate_tied_embedding(ids_n, dY, H, dL, c_true),
                               sum(c_true[i] * grads[i]["E"] for i in range(B)), rtol=1e-9, atol=1e-13)


def test_tied_embedding_special_cases_and_cross_term():
    B, T, M, d, V = 3, 7, 4, 5, 8
    ids = syn.zipf_ids(B, T, V, 1.1, 21)
    dY = syn.normal_f32((B, T, d), 1.0, 22)
    H = syn.normal_f32((B, M, d), 1.0, 23)
    dL = syn.normal_f32((B, M, V), 0.5, 24)
    zero = lambda a: np.zeros_like(a)
    # no output-projection gradient: the plain lookup; no lookup gradient: a dense layer with input dL, output gradient H
    np.testing.assert_allclose(orc.sqnorms_tied_embedding(ids, dY, H, zero(dL)), orc.sqnorms_embedding(ids, dY, V), rtol=1e-13)
    np.testing.assert_allclose(orc.sqnorms_tied_embedding(ids, zero(dY), H, dL), orc.sqnorms_dense(dL, H, False), rtol=1e-13)
    c = np.array([0.25, 1.0, 0.5])
    np.testing.assert_allclose(orc.clip_accumulate_tied_embedding(ids, dY, H, dL, c),
                               orc.clip_accumulate_embedding(ids, dY, c, V) + orc.clip_accumulate_dense(dL, H, c, False)[0],
                               rtol=1e-12, atol=1e-14)
    # entry by entry with plain loops, and the expansion of the square with its cross term
    n = orc.sqnorms_tied_embedding(ids, dY, H, dL)
    for i in range(B):
        tot = 0.0
        for v in range(V):
            for k in range(d):
                e = sum(float(dY[i, t, k]) for t in range(T) if ids[i, t] == v)
                e += sum(float(dL[i, m, v]) * float(H[i, m, k]) for m in range(M))
                tot += e * e
        assert abs(tot - n[i]) <= 1e-11 * tot
        cross = sum(float(dL[i, m, ids[i, t]]) * float(np.dot(dY[i, t].astype(np.float64), H[i, m].astype(np.float64)))
                    for t in range(T) for m in range(M))
        parts = orc.sqnorms_embedding(ids[i:i + 1], dY[i:i + 1], V)[0] + orc.sqnorms_dense(dL[i:i + 1], H[i:i + 1], False)[0]
        assert abs(parts + 2.0 * cross - n[i]) <= 1e-11 * n[i]
        assert abs(cross) > 1e-3 * n[i]                 # the cross term is not negligible in this case


def test_tied_embedding_square_table():
    """V == d: a transposed outer product would still have the right shape; autograd tells the two apart."""
    E = torch.arange(16, dtype=torch.float64).reshape(4, 4).requires_grad_(True) / 10.0
    E.retain_grad()
    ids = torch.tensor([[1, 3, 1]])
    x = E[ids]
    x.retain_grad()
    hm = torch.tanh(x[:, :2] * 0.7)
    hm.retain_grad()
    logits = hm @ E.T
    logits.retain_grad()
    (logits ** 2).sum().backward()
    npy = lambda t: t.detach().numpy().copy()
    g = orc.tied_embedding_example_grad(ids.numpy()[0].astype(np.int32), npy(x.grad)[0], npy(hm)[0], npy(logits.grad)[0])
    np.testing.assert_allclose(g, npy(E.grad), rtol=1e-12, atol=1e-14)


# ----------------------------------------------------------------------------------------------
# mega-batch accumulation
# ----------------------------------------------------------------------------------------------
def test_accumulation_is_linear_over_microbatches():
    A1, G1 = _c1_like(seed=20)
    A2, G2 = _c1_like(seed=30)
    L1 = [dict(kind="dense", A=A1, G=G1, has_bias=True)]
    L2 = [dict(kind="dense", A=A2, G=G2, has_bias=True)]
    s1, _, _ = orc.microbatch_clip_sum(L1, 1.0)
    s2, _, _ = orc.microbatch_clip_sum(L2, 1.0)
    acc, _, _ = orc.microbatch_clip_sum(L1, 1.0)
    acc, _, _ = orc.microbatch_clip_sum(L2, 1.0, acc)
    np.testing.assert_allclose(acc[0][0], s1[0][0] + s2[0][0], rtol=1e-13)
    np.testing.assert_allclose(acc[0][1], s1[0][1] + s2[0][1], rtol=1e-13)


# ----------------------------------------------------------------------------------------------
# bf16 widening
# ----------------------------------------------------------------------------------------------
def test_bf16_widening_matches_torch():
    x = syn.normal_f32((1000,), 3.0, 11)
    bits = syn.f32_to_bf16_bits(x)
    t = torch.from_numpy(x).to(torch.bfloat16)
    np.testing.assert_array_equal(orc.to_f64(bits), t.to(torch.float64).numpy())
    np.testing.assert_array_equal(bits, t.view(torch.int16).numpy().view(np.uint16))


# ----------------------------------------------------------------------------------------------
# Adam with decoupled weight decay
# ----------------------------------------------------------------------------------------------
def _table1():
    """Best-trial hyper-parameters as the paper prints them (Table 1; xi from Algorithm 1)."""
    import os

    vals = {}
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "table1_best_trial.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                vals[k] = float(v)
    return dict(lr=vals["learning_rate"], beta1=1 - vals["one_minus_beta1"], beta2=1 - vals["one_minus_beta2"],
                eps=vals["xi"], weight_decay=vals["weight_decay"])


HP = _table1()


def test_adamw_matches_torch_optim_five_steps():
    n = 257
    theta0 = syn.normal_f32((n,), 0.02, 12)
    p = torch.nn.Parameter(torch.from_numpy(theta0.astype(np.float64)))
    f32 = lambda x: float(np.float32(x))
    opt = torch.optim.AdamW([p], lr=f32(HP["lr"]), betas=(f32(HP["beta1"]), f32(HP["beta2"])), eps=f32(HP["eps"]),
                            weight_decay=f32(HP["weight_decay"]))
    th, m, v = theta0.astype(np.float64), np.zeros(n), np.zeros(n)
    Bsz = 64
    for t in range(1, 6):
        S = syn.normal_f32((n,), 5.0, 100 + t)
        p.grad = torch.from_numpy(S.astype(np.float64) / Bsz)
        opt.step()
        th, m, v, g = orc.noise_adamw(th, m, v, S, elem_offset=0, sigma=0.0, C=1.0, seed=0, step=t, batch_size=Bsz, **HP)
        np.testing.assert_allclose(th, p.detach().numpy(), rtol=1e-12, atol=1e-15)
    st = opt.state[p]
    np.testing.assert_allclose(m, st["exp_avg"].numpy(), rtol=1e-12)
    np.testing.assert_allclose(v, st["exp_avg_sq"].numpy(), rtol=1e-12)


def test_adamw_hand_worked_element():
    # theta=2, S=8, batch 4 -> g=2; beta1=.5, beta2=.75, t=1: m=1, v=1, mhat=2, vhat=4; xi=0.5:
    # theta' = 2 - 0.1*(2/(2+0.5) + 0.25*2) = 2 - 0.1*(0.8+0.5) = 1.87
    th, m, v, g = orc.noise_adamw(np.array([2.0]), np.zeros(1), np.zeros(1), np.array([8.0]), elem_offset=0, sigma=0.0,
                                  C=1.0, seed=0, step=1, batch_size=4, lr=0.1, beta1=0.5, beta2=0.75, eps=0.5,
                                  weight_decay=0.25)
    f = lambda x: float(np.float32(x))
    assert g[0] == 2.0 and m[0] == 1.0 and v[0] == 1.0
    assert math.isclose(th[0], 2 - f(0.1) * (0.8 + 0.5), rel_tol=1e-12)
    # second step from (m, v) with S = 0: m = .5, v = .75; mhat = .5/.75, vhat = .75/(1-.5625)
    th2, m2, v2, _ = orc.noise_adamw(th, m, v, np.zeros(1), elem_offset=0, sigma=0.0, C=1.0, seed=0, step=2,
                                     batch_size=4, lr=0.1, beta1=0.5, beta2=0.75, eps=0.5, weight_decay=0.25)
    mh, vh = 0.5 / 0.75, 0.75 / (1 - 0.5625)
    assert math.isclose(th2[0], th[0] - f(0.1) * (mh / (math.sqrt(vh) + 0.5) + 0.25 * th[0]), rel_tol=1e-12)


def test_adamw_zero_gradient_is_pure_decay():
    th, m, v, g = orc.noise_adamw(np.array([3.0], np.float32), np.zeros(1), np.zeros(1), np.zeros(1), elem_offset=0,
                                  sigma=0.0, C=1.0, seed=0, step=1, batch_size=8, **HP)
    f = lambda x: float(np.float32(x))
    assert math.isclose(th[0], 3.0 * (1 - f(HP["lr"]) * f(HP["weight_decay"])), rel_tol=1e-14)
    assert m[0] == 0 and v[0] == 0


# ----------------------------------------------------------------------------------------------
# Philox and the normal stream
# ----------------------------------------------------------------------------------------------
def _philox_bigint(ctr, key):
    """Independent scalar implementation with Python integers (written from the round definition)."""
    M0, M1, W0, W1 = 0xD2511F53, 0xCD9E8D57, 0x9E3779B9, 0xBB67AE85
    c = list(ctr)
    k = list(key)
    for r in range(10):
        p0, p1 = M0 * c[0], M1 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & 0xFFFFFFFF, (p0 >> 32) ^ c[3] ^ k[1], p0 & 0xFFFFFFFF]
        k = [(k[0] + W0) & 0xFFFFFFFF, (k[1] + W1) & 0xFFFFFFFF]
    return c


def _philox_inverse(out, key):
    """Run the ten rounds backwards: needs the modular inverses of the (odd) multipliers, so it is a
    different computation from the forward rounds, and only the true bijection survives it."""
    M0, M1, W0, W1 = 0xD2511F53, 0xCD9E8D57, 0x9E3779B9, 0xBB67AE85
    M0i, M1i = pow(M0, -1, 1 << 32), pow(M1, -1, 1 << 32)
    keys = [((key[0] + r * W0) & 0xFFFFFFFF, (key[1] + r * W1) & 0xFFFFFFFF) for r in range(10)]
    c = list(out)
    for r in reversed(range(10)):
        k0, k1 = keys[r]
        lo1, lo0 = c[1], c[3]
        c0 = (lo0 * M0i) & 0xFFFFFFFF  # lo0 = (M0*c0) mod 2^32
        c2 = (lo1 * M1i) & 0xFFFFFFFF
        hi0, hi1 = (M0 * c0) >> 32, (M1 * c2) >> 32
        c1 = c[0] ^ hi1 ^ k0
        c3 = c[2] ^ hi0 ^ k1
        c = [c0, c1, c2, c3]
    return c


def test_philox_against_bigint_and_inverse():
    rng = np.random.default_rng(13)
    cases = [(0, 0, 0), (1, 0, 1), (2 ** 32 - 1, 7, 1), (2 ** 32, 0xDEADBEEFCAFEF00D, 2 ** 33 + 5)]
    cases += [(int(rng.integers(0, 2 ** 40)), int(rng.integers(0, 2 ** 63)), int(rng.integers(1, 2 ** 40))) for _ in range(20)]
    for blk, seed, step in cases:
        w = orc.philox_u32(4, 4 * blk, seed, step)
        ctr = [blk & 0xFFFFFFFF, blk >> 32, step & 0xFFFFFFFF, step >> 32]
        key = [seed & 0xFFFFFFFF, seed >> 32]
        ref = _philox_bigint(ctr, key)
        assert [int(x) for x in w] == ref
        assert _philox_inverse(ref, key) == ctr


def test_philox_mapping_and_slicing():
    full = orc.philox_u32(64, 0, 99, 3)
    for off, n in [(0, 1), (1, 6), (3, 2), (4, 4), (5, 59), (63, 1)]:
        np.testing.assert_array_equal(orc.philox_u32(n, off, 99, 3), full[off:off + n])
    assert not np.array_equal(orc.philox_u32(64, 0, 99, 4), full)   # step changes the stream
    assert not np.array_equal(orc.philox_u32(64, 0, 98, 3), full)   # seed changes the stream
    # the high seed word and the high step word matter
    assert not np.array_equal(orc.philox_u32(8, 0, 99 + (1 << 32), 3), full[:8])
    assert not np.array_equal(orc.philox_u32(8, 0, 99, 3 + (1 << 32)), full[:8])
    # block index crosses 2^32
    a = orc.philox_u32(8, 4 * (2 ** 32) - 4, 5, 1)
    b = orc.philox_u32(4, 4 * (2 ** 32), 5, 1)
    np.testing.assert_array_equal(a[4:], b)
    assert not np.array_equal(orc.philox_u32(4, 0, 5, 1), b)


def test_philox_statistics():
    w = orc.philox_u32(1 << 20, 0, 1234, 1)
    bits = np.unpackbits(w.view(np.uint8))
    assert abs(bits.mean() - 0.5) < 5 * 0.5 / math.sqrt(bits.size)
    blocks = w.reshape(-1, 4)
    assert len(np.unique(blocks, axis=0)) == blocks.shape[0]
    # avalanche: consecutive counters differ in about half of the 128 output bits
    x = np.unpackbits((blocks[1:] ^ blocks[:-1]).view(np.uint8), axis=1).sum(axis=1)
    assert abs(x.mean() - 64) < 0.1 and 20 < x.min() and x.max() < 108


def test_uniforms_exact_in_fp32_and_open_interval():
    r = np.array([0, 1, 511, 512, 2 ** 31, 2 ** 32 - 1], dtype=np.uint32)
    u = orc.uniform_from_u32(r)
    assert u.min() == 2.0 ** -24 and u.max() == 1 - 2.0 ** -24
    np.testing.assert_array_equal(u.astype(np.float32).astype(np.float64), u)
    assert u[2] == u[0] and u[3] == 1.5 * 2.0 ** -23


def test_box_muller_structure():
    n = 1 << 12
    w = orc.philox_u32(n, 0, 7, 2).reshape(-1, 2)
    z = orc.normals(n, 0, 7, 2).reshape(-1, 2)
    u0, u1 = orc.uniform_from_u32(w[:, 0]), orc.uniform_from_u32(w[:, 1])
    np.testing.assert_allclose((z ** 2).sum(axis=1), -2 * np.log(u0), rtol=1e-12)
    ang = np.mod(np.arctan2(z[:, 1], z[:, 0]), 2 * np.pi)
    np.testing.assert_allclose(ang, 2 * np.pi * u1, rtol=1e-9, atol=1e-12)
    # slices of the element space see the same normals
    np.testing.assert_array_equal(orc.normals(37, 5, 7, 2), z.reshape(-1)[5:42])


def test_normal_moments_and_ks():
    from scipy import stats

    N = 1 << 22
    z = orc.normals(N, 0, 1234, 1)
    assert abs(z.mean()) < 5 / math.sqrt(N)
    assert abs(z.var() - 1) < 5 * math.sqrt(2 / N)
    assert abs(stats.kurtosis(z, fisher=False) - 3) < 5 * math.sqrt(24 / N)
    assert abs(stats.skew(z)) < 5 * math.sqrt(6 / N)
    assert np.abs(z).max() <= math.sqrt(-2 * math.log(2.0 ** -24)) + 1e-12
    assert stats.kstest(z[: 1 << 18], "norm").pvalue > 1e-4
    # even/odd elements (cos/sin branches) are uncorrelated
    assert abs(np.corrcoef(z[0::2], z[1::2])[0, 1]) < 5 / math.sqrt(N / 2)


def test_noise_scale_on_the_mean_gradient():
    n, Bsz, sigma, C = 1 << 18, 4096, 0.6, 0.5
    _, m, _, g = orc.noise_adamw(np.zeros(n), np.zeros(n), np.zeros(n), np.zeros(n), elem_offset=0, sigma=sigma, C=C,
                                 seed=1234, step=1, batch_size=Bsz, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-11,
                                 weight_decay=0.5)
    f = lambda x: float(np.float32(x))
    zrec = g * Bsz / (f(sigma) * f(C))
    assert abs(zrec.std() - 1) < 5 / math.sqrt(2 * n)
    np.testing.assert_allclose(m / (1 - f(0.9)), g, rtol=1e-12)
    np.testing.assert_allclose(zrec, orc.normals(n, 0, 1234, 1), rtol=1e-9, atol=1e-12)


def test_noise_depends_on_global_element_index():
    n = 64
    S = syn.normal_f32((n,), 1.0, 14)
    kw = dict(sigma=1.0, C=1.0, seed=0, step=1, batch_size=32, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-11, weight_decay=0.01)
    full = orc.noise_adamw(np.zeros(n), np.zeros(n), np.zeros(n), S, elem_offset=0, **kw)
    part = orc.noise_adamw(np.zeros(10), np.zeros(10), np.zeros(10), S[13:23], elem_offset=13, **kw)
    for a, b in zip(full, part):
        np.testing.assert_array_equal(a[13:23], b)


# ----------------------------------------------------------------------------------------------
# gradient signal-to-noise ratio (Section 5.2.1, effect of batch size on DP gradients)
# ----------------------------------------------------------------------------------------------
def test_gradient_snr_closed_forms():
    n, sigma, C = 1 << 16, 0.6, 0.5
    f = lambda x: float(np.float32(x))
    S = np.full(n, 0.25)
    sig, noi = orc.gradient_snr_terms(S, elem_offset=8, sigma=sigma, C=C, seed=7, step=3)
    assert sig == n * 0.0625                                    # constant vector: n a^2, exact in binary
    # chi-square with n degrees of freedom: mean n, standard deviation sqrt(2n)
    assert abs(noi / (f(sigma) * f(C)) ** 2 - n) < 5 * math.sqrt(2 * n)
    # sigma scales the noise norm linearly, C likewise; the signal does not move
    sig2, noi2 = orc.gradient_snr_terms(S, elem_offset=8, sigma=2 * sigma, C=C, seed=7, step=3)
    assert sig2 == sig and math.isclose(noi2, 4 * noi, rel_tol=1e-12)
    _, noi3 = orc.gradient_snr_terms(S, elem_offset=8, sigma=sigma, C=2 * C, seed=7, step=3)
    assert math.isclose(noi3, 4 * noi, rel_tol=1e-12)
    assert orc.gradient_snr_terms(S, elem_offset=8, sigma=0.0, C=C, seed=7, step=3) == (sig, 0.0)
    # expected ratio for a constant signal: a sqrt(n) / (sigma C sqrt(n)) = a / (sigma C), within the chi-square spread
    assert math.isclose(orc.gradient_snr(sig, noi), 0.25 / (f(sigma) * f(C)), rel_tol=5 / math.sqrt(2 * n))
    assert orc.gradient_snr(9.0, 4.0) == 1.5 and orc.gradient_snr(1.0, 0.0) == float("inf")


def test_gradient_snr_noise_is_what_the_update_adds():
    """The noise norm is the norm of the vector the update actually adds to the sum: recover it from the
    update's own gradient, g*|B| - S, for a slice that starts inside a Philox block."""
    n, off, Bsz = 1001, 13, 64
    S = syn.normal_f32((n,), 3.0, 21)
    kw = dict(elem_offset=off, sigma=0.8, C=0.7, seed=99, step=5)
    _, _, _, g = orc.noise_adamw(np.zeros(n), np.zeros(n), np.zeros(n), S, batch_size=Bsz, lr=1e-3, beta1=0.9, beta2=0.999,
                                 eps=1e-11, weight_decay=0.0, **kw)
    added = g * Bsz - S.astype(np.float64)
    sig, noi = orc.gradient_snr_terms(S, **kw)
    assert math.isclose(noi, float(np.dot(added, added)), rel_tol=1e-9)
    assert math.isclose(sig, float(np.linalg.norm(S.astype(np.float64)) ** 2), rel_tol=1e-12)
    # slices add up (squared norms are additive over a partition of the element range)
    a = orc.gradient_snr_terms(S[:333], **kw)
    b = orc.gradient_snr_terms(S[333:], **dict(kw, elem_offset=off + 333))
    assert math.isclose(a[0] + b[0], sig, rel_tol=1e-12) and math.isclose(a[1] + b[1], noi, rel_tol=1e-12)


def test_gradient_snr_grows_with_batch_size():
    """Section 5.2.1's observation in its simplest form: with per-example clipped gradients pointing the same
    way, the signal norm grows like |B| while the noise norm does not depend on |B|."""
    n = 4096
    unit = syn.normal_f32((n,), 1.0, 31).astype(np.float64)
    unit /= np.linalg.norm(unit)
    snr = []
    for Bsz in (64, 256, 1024):
        sig, noi = orc.gradient_snr_terms(Bsz * unit, elem_offset=0, sigma=1.0, C=1.0, seed=1, step=1)
        snr.append(orc.gradient_snr(sig, noi))
    assert math.isclose(snr[1] / snr[0], 4.0, rel_tol=1e-9) and math.isclose(snr[2] / snr[1], 4.0, rel_tol=1e-9)
    assert math.isclose(snr[0], 64 / math.sqrt(n), rel_tol=0.1)


# ----------------------------------------------------------------------------------------------
# schedules (batch sizes q_t of the batch-size study; learning rates eta_t of the tuning section)
# ----------------------------------------------------------------------------------------------
def _schedule_numbers():
    out = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "batch_size_schedule.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, val = line.split()
                out[k] = int(val)
    return out


def test_batch_size_schedule_reproduces_the_papers_numbers():
    n = _schedule_numbers()
    q = lambda t: orc.batch_size_schedule(t, n["b_start"], n["b_end"], n["ramp_steps"], n["parts"])
    assert q(1) == 262144 and q(n["ramp_steps"] + 1) == 1048576 and q(20000) == 1048576
    quarter = n["ramp_steps"] // n["parts"]
    sizes = [q(k * quarter + 1) for k in range(n["parts"] + 1)]
    jumps = np.diff(sizes)
    assert (jumps == jumps[0]).all() and abs(int(jumps[0]) - n["jump_approx"]) < 1000      # "~196k" each quarter
    assert sizes == [262144, 458752, 655360, 851968, 1048576]                                # 2^18 + k * 3 * 2^16
    # constant within a quarter; the jump comes after the quarter's last step, never earlier
    assert q(quarter) == sizes[0] and q(quarter + 1) == sizes[1] and q(n["ramp_steps"]) == sizes[3]
    all_q = np.array([q(t) for t in range(1, n["ramp_steps"] + 2)])
    assert (np.diff(all_q) >= 0).all() and len(set(all_q.tolist())) == 5
    # examples visited over the ramp against a fixed 1M batch: the mean of the four plateaus
    assert all_q[:-1].sum() == quarter * sum(sizes[:4])


def test_batch_size_schedule_general_and_errors():
    # ragged: 10 -> 20 in 3 jumps over 7 steps; jumps of 3 after floor-boundaries 7/3, 14/3; ends exactly at 20
    got = [orc.batch_size_schedule(t, 10, 20, 7, 3) for t in range(1, 10)]
    assert got == [10, 10, 10, 13, 13, 16, 16, 20, 20]
    assert orc.batch_size_schedule(5, 64, 64, 4, 2) == 64
    for bad in ((0, 1, 2, 4, 2), (1, 1, 2, 4, 0), (1, 3, 2, 4, 2), (1, 1, 2, 1, 2)):
        with pytest.raises(ValueError):
            orc.batch_size_schedule(*bad)


def test_lr_schedule_shape():
    n = _schedule_numbers()
    W, Ttot, peak = n["warmup_steps"], n["total_steps"], HP["lr"]
    lr = np.array([orc.lr_schedule(t, peak, W, Ttot) for t in range(1, Ttot + 2)])
    assert lr[W - 1] == peak and lr.argmax() == W - 1            # the peak is reached exactly at the end of warm-up
    np.testing.assert_allclose(np.diff(lr[:W]), peak / W, rtol=1e-9)             # linear: constant first difference
    d2 = np.diff(lr[W - 1:Ttot], 2)
    np.testing.assert_allclose(d2, 2 * peak / (Ttot - W) ** 2, rtol=1e-6)        # quadratic: constant second difference
    assert lr[Ttot - 1] == 0.0 and lr[Ttot] == 0.0 and (lr >= 0).all()
    assert math.isclose(lr[(W + Ttot) // 2 - 1], peak / 4, rel_tol=1e-12)        # half-way down the decay: a quarter
    assert orc.lr_schedule(1, peak, 0, 10) == peak * (9 / 10) ** 2               # no warm-up: decay from step 0
    with pytest.raises(ValueError):
        orc.lr_schedule(0, peak, W, Ttot)
    with pytest.raises(ValueError):
        orc.lr_schedule(1, peak, 10, 5)


# ----------------------------------------------------------------------------------------------
# privacy accounting (Renyi DP of the sampled Gaussian mechanism, composed over a batch-size schedule)
# ----------------------------------------------------------------------------------------------
def _renyi_by_quadrature(q, sigma, alpha):
    """The definition itself: D_alpha(P || Q) = ln E_Q[(P/Q)^alpha] / (alpha - 1) with Q = N(0, sigma^2) and
    P = (1-q) N(0, sigma^2) + q N(1, sigma^2) (one example changes the clipped, C-normalised sum by at most 1),
    by the trapezoid rule on a fine grid."""
    x = np.linspace(-40.0 * sigma, 40.0 * sigma + alpha, 2_000_001)
    logQ = -0.5 * (x / sigma) ** 2
    ratio = (1.0 - q) + q * np.exp((2.0 * x - 1.0) / (2.0 * sigma * sigma))      # P/Q pointwise
    integrand = np.exp(logQ + alpha * np.log(ratio)) / (sigma * math.sqrt(2.0 * math.pi))
    return math.log(np.trapezoid(integrand, x)) / (alpha - 1)


def test_rdp_matches_the_definition_by_quadrature():
    for q, sigma, alpha in [(0.01, 0.6, 2), (0.01, 0.6, 5), (0.3, 1.0, 3), (0.003, 0.8, 16), (1.0, 1.5, 4), (0.5, 2.0, 9)]:
        assert math.isclose(orc.rdp_sampled_gaussian(q, sigma, alpha), _renyi_by_quadrature(q, sigma, alpha), rel_tol=1e-7)


def test_rdp_closed_forms():
    # no subsampling: the Gaussian mechanism, alpha / (2 sigma^2)
    for sigma, alpha in [(0.6, 2), (1.0, 7), (2.5, 64)]:
        assert math.isclose(orc.rdp_sampled_gaussian(1.0, sigma, alpha), alpha / (2 * sigma * sigma), rel_tol=1e-13)
    # order 2 by hand: ln(1 + q^2 (e^{1/sigma^2} - 1))
    for q, sigma in [(0.01, 1.0), (0.25, 0.7)]:
        assert math.isclose(orc.rdp_sampled_gaussian(q, sigma, 2), math.log1p(q * q * math.expm1(1 / sigma ** 2)), rel_tol=1e-12)
    assert orc.rdp_sampled_gaussian(0.0, 1.0, 8) == 0.0                      # nothing sampled: nothing revealed
    # monotone in the sampling rate, the order and 1/sigma
    e = [orc.rdp_sampled_gaussian(q, 0.8, 8) for q in (1e-4, 1e-3, 1e-2, 1e-1, 1.0)]
    assert all(a < b for a, b in zip(e, e[1:]))
    e = [orc.rdp_sampled_gaussian(0.01, 0.8, a) for a in (2, 3, 8, 32)]
    assert all(a < b for a, b in zip(e, e[1:]))
    assert orc.rdp_sampled_gaussian(0.01, 0.5, 8) > orc.rdp_sampled_gaussian(0.01, 1.0, 8)
    for bad in ((-0.1, 1.0, 2), (1.1, 1.0, 2), (0.1, 0.0, 2), (0.1, 1.0, 1)):
        with pytest.raises(ValueError):
            orc.rdp_sampled_gaussian(*bad)


def test_rdp_epsilon_composition_over_a_batch_size_schedule():
    n = _schedule_numbers()
    N, sigma, delta = 346_000_000, 0.6, 2.89e-9          # data-set size and delta as the paper states them (delta = 1/N)
    sizes = [orc.batch_size_schedule(k * 1875 + 1, n["b_start"], n["b_end"], n["ramp_steps"], n["parts"]) for k in range(5)]
    q = [b / N for b in sizes]
    steps = [1875, 1875, 1875, 1875, n["total_steps"] - n["ramp_steps"]]
    eps, alpha = orc.rdp_epsilon(q, steps, sigma, delta, 64)
    # the definition of the conversion at the reported order, from the per-step values
    rdp = sum(s * orc.rdp_sampled_gaussian(qq, sigma, alpha) for qq, s in zip(q, steps))
    assert math.isclose(eps, rdp + math.log(1 / delta) / (alpha - 1), rel_tol=1e-12)
    # no other order does better; splitting a phase in two changes nothing; the schedule sits between its extremes
    for a in range(2, 65):
        r = sum(s * orc.rdp_sampled_gaussian(qq, sigma, a) for qq, s in zip(q, steps))
        assert eps <= r + math.log(1 / delta) / (a - 1) + 1e-12
    eps_split, _ = orc.rdp_epsilon(q + [q[-1]], steps[:-1] + [5000, steps[-1] - 5000], sigma, delta, 64)
    assert math.isclose(eps, eps_split, rel_tol=1e-12)
    lo, _ = orc.rdp_epsilon([q[0]], [n["total_steps"]], sigma, delta, 64)
    hi, _ = orc.rdp_epsilon([q[-1]], [n["total_steps"]], sigma, delta, 64)
    assert lo < eps < hi
    # a single Gaussian release (q = 1, one step): min over alpha of alpha/(2 sigma^2) + ln(1/delta)/(alpha-1), on integers
    e1, a1 = orc.rdp_epsilon([1.0], [1], 4.0, 1e-5, 256)
    ref = min(a / 32.0 + math.log(1e5) / (a - 1) for a in range(2, 257))
    assert math.isclose(e1, ref, rel_tol=1e-12) and abs(a1 - (1 + math.sqrt(32 * math.log(1e5)))) <= 1


def test_rdp_noise_multiplier_inverts_the_guarantee():
    """The search for sigma against what fixes it: the unsampled Gaussian mechanism, whose guarantee is typed out here
    (n alpha / (2 sigma^2) + ln(1/delta) / (alpha - 1), best integer order) and strictly decreases in sigma, so the
    smallest sigma that meets eps(sigma0) is sigma0 itself; then, on the paper's batch-size schedule, that the result
    meets the target, that nothing 3 tolerances smaller does, and the directions in which it must move."""
    def eps_plain(sigma, n, delta, max_alpha):
        return min(n * a / (2 * sigma * sigma) + math.log(1 / delta) / (a - 1) for a in range(2, max_alpha + 1))

    for sigma0, n, delta in [(4.0, 1, 1e-5), (30.0, 100, 1e-6), (0.9, 1, 1e-3), (1.0, 1, 1e-5), (2.0, 7, 1e-4)]:
        target = eps_plain(sigma0, n, delta, 64)
        got = orc.rdp_noise_multiplier([1.0], [n], target, delta, 64, 1e-7)
        assert sigma0 * (1 - 1e-9) <= got <= sigma0 * (1 + 2e-7), (sigma0, got)
        assert eps_plain(got, n, delta, 64) <= target * (1 + 1e-12)

    n = _schedule_numbers()
    N, delta = 346_000_000, 2.89e-9
    sizes = [orc.batch_size_schedule(k * 1875 + 1, n["b_start"], n["b_end"], n["ramp_steps"], n["parts"]) for k in range(5)]
    q = [b / N for b in sizes]
    steps = [1875, 1875, 1875, 1875, n["total_steps"] - n["ramp_steps"]]
    tol = 1e-4
    sig = {t: orc.rdp_noise_multiplier(q, steps, t, delta, 32, tol) for t in (2.0, 5.36, 10.6)}
    for t, s in sig.items():
        assert orc.rdp_epsilon(q, steps, s, delta, 32)[0] <= t                       # meets the target
        assert orc.rdp_epsilon(q, steps, s * (1 - 3 * tol), delta, 32)[0] > t        # and is the smallest that does
    assert sig[2.0] > sig[5.36] > sig[10.6]                                          # a tighter target needs more noise
    longer = orc.rdp_noise_multiplier(q, [2 * k for k in steps], 5.36, delta, 32, tol)
    assert longer > sig[5.36]                                                        # and so do more steps
    # below the conversion term of the largest order no sigma helps; with no steps any sigma does
    with pytest.raises(ValueError):
        orc.rdp_noise_multiplier(q, steps, 0.9 * math.log(1 / delta) / 31, delta, 32, tol)
    assert orc.rdp_noise_multiplier([0.1], [0], 1.0, 1e-5, 32, tol) <= 2.0 ** -9
    for bad in ((0.0, 1e-4), (1.0, 0.0), (1.0, 1.0)):
        with pytest.raises(ValueError):
            orc.rdp_noise_multiplier(q, steps, bad[0], delta, 32, bad[1])


# ----------------------------------------------------------------------------------------------
# stored reference (written by tests/golden/make_oracle_reference.py from the oracle alone): drift guard
# ----------------------------------------------------------------------------------------------
def test_oracle_matches_its_stored_reference():
    import importlib.util
    import json
    import os

    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    spec = importlib.util.spec_from_file_location("make_oracle_reference", os.path.join(here, "make_oracle_reference.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    now = mod.build()
    ref = json.load(open(os.path.join(here, "oracle_c1_reference.json")))
    assert set(now) == set(ref)
    for k in ref:
        if k.startswith("philox") or k == "sum_idx":
            assert now[k] == ref[k], k
        else:
            np.testing.assert_allclose(now[k], ref[k], rtol=1e-12, atol=1e-300, err_msg=k)
