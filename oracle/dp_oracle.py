"""CPU oracle for the per-example clipped-gradient step of DP-SGD with Adam and
decoupled weight decay (Algorithm 1 of the paper, the g_t line through the theta_t line).

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this module; only
tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg do.  It shares no code
with the HIP path: its own bf16 widening, its own Philox, its own loops.

What it computes, written out as the plain definition (numpy, fp64 arithmetic):
for every example, every per-example gradient array is MATERIALISED explicitly
(dense: A_i^T G_i and the column sums of G_i, following the outer-product form of a
fully connected layer's gradient given in the scale-invariance section; LayerNorm
gain/offset; embedding rows), the squared L2 norm over ALL of the example's parameter
gradients is taken, the clip factor min(1, C/norm) is formed, and the clip-weighted
gradients are summed.  No Gram identity, no flattened GEMM over the batch: those are
what the GPU path uses and what this oracle is there to check.

Readings of points the paper leaves open (each also listed in the design notes):
  * clip(g, C) = g * min(1, C/||g||_2) with the global norm over all tensors; ||g|| = 0 -> factor 1.
  * the decay term of the update line uses theta_{t-1} (decoupled weight decay), times eta_t.
  * xi sits outside the square root, after bias correction.
  * the divisor |B_t| is the mega-batch example count; noise is added once, before dividing.
  * noise: Philox4x32-10 (Salmon et al., SC'11) keyed by (seed), counter (element block, step),
    23-bit uniforms u = ((r >> 9) + 1/2) * 2^-23 (exact in fp32), Box-Muller on word pairs.

Pins (tests/test_oracle_pins.py): brute-force autograd on a tiny BERT-like model for the
gradient formulas, norms, clip factors and sums (a second tiny model, with its output projection tied
to the lookup table, for tied_embedding_example_grad); closed forms (T = 1, rank one); clip
invariant and clip no-op against a flat GEMM / bincount / index_add; torch.optim.AdamW and a
hand-worked element for the update; statistical moments and exact-uniform checks for the
normals; for the privacy accounting, quadrature of the Renyi divergence's definition, closed forms, and
for the noise-multiplier search the unsampled Gaussian mechanism (whose guarantee the test types out) plus
minimality of the result.  Philox known-answer vectors are NOT in this repository: its raw stream is
"parity unpinned" on the CPU beyond an independent big-integer implementation, the
inverse-round bijection check and avalanche statistics.  The gpu-marked test
test_philox_matches_rocrand_host_generator pins the words bit for bit against rocRAND's host
Philox4x32-10 generator, an independent implementation that only runs where a GPU is present.
"""
from __future__ import annotations

import numpy as np

# --------------------------------------------------------------------------------------
# input widening
# --------------------------------------------------------------------------------------


def to_f64(x: np.ndarray) -> np.ndarray:
    """fp32/fp64 arrays are widened; uint16 arrays are bf16 bit patterns (sign, 8 exponent,
    7 mantissa bits = the top half of an fp32) and are widened exactly."""
    x = np.asarray(x)
    if x.dtype == np.uint16:
        return (x.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    if x.dtype in (np.float32, np.float64):
        return x.astype(np.float64)
    raise TypeError(f"unsupported input dtype {x.dtype}")


# --------------------------------------------------------------------------------------
# per-example gradients, materialised (one example at a time)
# --------------------------------------------------------------------------------------


def dense_example_grads(A_i: np.ndarray, G_i: np.ndarray):
    """Dense layer y = xW + b, W in R^{d_in x d_out}.  A_i [T, d_in] are the layer inputs of one
    example, G_i [T, d_out] the gradient of that example's loss w.r.t. the layer outputs.
    Gradient of W: sum over tokens of outer(a_t, g_t) = A_i^T G_i; gradient of b: sum_t g_t."""
    A_i = to_f64(A_i)
    G_i = to_f64(G_i)
    gW = A_i.T @ G_i
    gb = G_i.sum(axis=0)
    return gW, gb


def layernorm_example_grads(X_i: np.ndarray, G_i: np.ndarray):
    """LayerNorm y = gamma * xhat + beta.  X_i [T, d] are the normalised activations xhat."""
    X_i = to_f64(X_i)
    G_i = to_f64(G_i)
    return (G_i * X_i).sum(axis=0), G_i.sum(axis=0)


def embedding_example_grad(ids_i: np.ndarray, G_i: np.ndarray, V: int):
    """Embedding lookup y_t = E[id_t].  Returns (rows, R): the sorted distinct ids of the example and
    the explicit gradient rows R[k] = sum_{t: id_t = rows[k]} g_t (all other rows of the V x d
    gradient are zero)."""
    ids_i = np.asarray(ids_i)
    if ids_i.min(initial=0) < 0 or ids_i.max(initial=0) >= V:
        raise IndexError("token id out of range")
    G_i = to_f64(G_i)
    rows, inv = np.unique(ids_i, return_inverse=True)
    R = np.zeros((rows.shape[0], G_i.shape[1]), dtype=np.float64)
    for t in range(ids_i.shape[0]):
        R[inv[t]] += G_i[t]
    return rows, R


def embedding_example_grad_dense(ids_i, G_i, V):
    rows, R = embedding_example_grad(ids_i, G_i, V)
    E = np.zeros((V, R.shape[1]), dtype=np.float64)
    E[rows] = R
    return E


def tied_embedding_example_grad(ids_i, dY_i, H_i, dL_i):
    """A table E [V, d] that one example uses twice: as the lookup y_t = E[ids_t] of its T tokens (Section
    4.3's word-piece table) and as the output projection logits = H_i E^T of M selected positions (the
    masked-token head of BERT; the paper does not say whether its model ties the two, this is the gradient if it
    does).  E is ONE parameter, so the example has ONE gradient for it, the sum of both uses:
    the rows dY_i scattered to their ids, plus the outer-product form dL_i^T H_i of a fully connected layer whose
    weight is E^T (input H_i [M, d], output gradient dL_i [M, V]).  Returned as the explicit [V, d] array."""
    dL_i = to_f64(dL_i)
    H_i = to_f64(H_i)
    V = dL_i.shape[1]
    g = embedding_example_grad_dense(ids_i, dY_i, V)
    for m in range(dL_i.shape[0]):
        g += np.outer(dL_i[m], H_i[m])
    return g


# --------------------------------------------------------------------------------------
# pass 1: per-example squared norms of one layer
# --------------------------------------------------------------------------------------


def sqnorms_dense(A, G, has_bias: bool) -> np.ndarray:
    B = A.shape[0]
    n = np.zeros(B, dtype=np.float64)
    for i in range(B):
        gW, gb = dense_example_grads(A[i], G[i])
        n[i] = np.sum(gW * gW)
        if has_bias:
            n[i] += np.sum(gb * gb)
    return n


def sqnorms_layernorm(X, G) -> np.ndarray:
    B = X.shape[0]
    n = np.zeros(B, dtype=np.float64)
    for i in range(B):
        gg, gb = layernorm_example_grads(X[i], G[i])
        n[i] = np.sum(gg * gg) + np.sum(gb * gb)
    return n


def sqnorms_embedding(ids, G, V: int) -> np.ndarray:
    B = ids.shape[0]
    n = np.zeros(B, dtype=np.float64)
    for i in range(B):
        _, R = embedding_example_grad(ids[i], G[i], V)
        n[i] = np.sum(R * R)
    return n


def sqnorms_tied_embedding(ids, dY, H, dL) -> np.ndarray:
    B = ids.shape[0]
    n = np.zeros(B, dtype=np.float64)
    for i in range(B):
        g = tied_embedding_example_grad(ids[i], dY[i], H[i], dL[i])
        n[i] = np.sum(g * g)
    return n


# --------------------------------------------------------------------------------------
# clip factor
# --------------------------------------------------------------------------------------


def clip_factors(sqnorms: np.ndarray, C: float) -> np.ndarray:
    """c_i = min(1, C / ||g_i||); a zero gradient is left alone (factor 1)."""
    n = np.asarray(sqnorms, dtype=np.float64)
    c = np.ones_like(n)
    pos = n > 0
    c[pos] = np.minimum(1.0, float(C) / np.sqrt(n[pos]))
    return c


# --------------------------------------------------------------------------------------
# pass 2: clip-weighted sums of one layer
# --------------------------------------------------------------------------------------


def clip_accumulate_dense(A, G, c, has_bias: bool):
    B = A.shape[0]
    S_W = np.zeros((A.shape[2], G.shape[2]), dtype=np.float64)
    S_b = np.zeros(G.shape[2], dtype=np.float64)
    for i in range(B):
        gW, gb = dense_example_grads(A[i], G[i])
        S_W += c[i] * gW
        S_b += c[i] * gb
    return S_W, (S_b if has_bias else None)


def clip_accumulate_dense_entries(A_cols, G_cols, c) -> np.ndarray:
    """Selected entries of the clip-weighted dense sum, one by one: A_cols[i, t, k] = A[i, t, p_k] and
    G_cols[i, t, k] = G[i, t, q_k] for the k-th sampled entry (p_k, q_k).  For every example the entry
    of its own gradient, sum_t A[i,t,p] G[i,t,q], is formed explicitly and added with weight c_i.
    (For full-size workloads, where the whole d_in x d_out sum is out of the oracle's reach.)"""
    A_cols = to_f64(A_cols)
    G_cols = to_f64(G_cols)
    out = np.zeros(A_cols.shape[2], dtype=np.float64)
    for i in range(A_cols.shape[0]):
        entry_i = np.sum(A_cols[i] * G_cols[i], axis=0)
        out += c[i] * entry_i
    return out


def clip_accumulate_layernorm(X, G, c):
    d = X.shape[2]
    S_g = np.zeros(d, dtype=np.float64)
    S_b = np.zeros(d, dtype=np.float64)
    for i in range(X.shape[0]):
        gg, gb = layernorm_example_grads(X[i], G[i])
        S_g += c[i] * gg
        S_b += c[i] * gb
    return S_g, S_b


def clip_accumulate_embedding(ids, G, c, V: int):
    S_E = np.zeros((V, G.shape[2]), dtype=np.float64)
    for i in range(ids.shape[0]):
        rows, R = embedding_example_grad(ids[i], G[i], V)
        S_E[rows] += c[i] * R
    return S_E


def clip_accumulate_tied_embedding(ids, dY, H, dL, c):
    S_E = np.zeros((dL.shape[2], dY.shape[2]), dtype=np.float64)
    for i in range(ids.shape[0]):
        S_E += c[i] * tied_embedding_example_grad(ids[i], dY[i], H[i], dL[i])
    return S_E


# --------------------------------------------------------------------------------------
# one micro-batch over a whole manifest of layers
# --------------------------------------------------------------------------------------


def _layer_example_grads(layer: dict, i: int):
    k = layer["kind"]
    if k == "dense":
        gW, gb = dense_example_grads(layer["A"][i], layer["G"][i])
        return [gW, gb] if layer.get("has_bias", False) else [gW]
    if k == "layernorm":
        gg, gb = layernorm_example_grads(layer["X"][i], layer["G"][i])
        return [gg, gb]
    if k == "embedding":
        return [embedding_example_grad(layer["ids"][i], layer["G"][i], layer["V"])]
    if k == "tied_embedding":  # "G" is the gradient of the lookup's output (dY)
        return [tied_embedding_example_grad(layer["ids"][i], layer["G"][i], layer["H"][i], layer["dL"][i])]
    raise ValueError(k)


def microbatch_sqnorms(layers: list, examples=None) -> np.ndarray:
    """Squared global gradient norm of each example: the sum over every layer of the manifest."""
    B = layers[0]["G"].shape[0]
    examples = range(B) if examples is None else examples
    out = []
    for i in examples:
        n_i = 0.0
        for layer in layers:
            for g in _layer_example_grads(layer, i):
                if isinstance(g, tuple):
                    g = g[1]
                n_i += float(np.sum(g * g))
        out.append(n_i)
    return np.asarray(out, dtype=np.float64)


def microbatch_clip_sum(layers: list, C: float, sums: list | None = None):
    """The sum over the micro-batch of clip(grad_i, C), per tensor.

    Returns (sums, sqnorms, c): `sums` is a list (one entry per layer) of lists of fp64 arrays in
    the tensor order of the manifest; pass the previous call's `sums` to accumulate a mega-batch."""
    B = layers[0]["G"].shape[0]
    if sums is None:
        sums = []
        for layer in layers:
            k = layer["kind"]
            if k == "dense":
                d_in, d_out = layer["A"].shape[2], layer["G"].shape[2]
                s = [np.zeros((d_in, d_out))]
                if layer.get("has_bias", False):
                    s.append(np.zeros(d_out))
            elif k == "layernorm":
                d = layer["G"].shape[2]
                s = [np.zeros(d), np.zeros(d)]
            else:
                s = [np.zeros((layer["V"], layer["G"].shape[2]))]
            sums.append(s)
    sq = np.zeros(B)
    cs = np.zeros(B)
    for i in range(B):
        grads = [_layer_example_grads(layer, i) for layer in layers]
        n_i = 0.0
        for gl in grads:
            for g in gl:
                if isinstance(g, tuple):
                    g = g[1]
                n_i += float(np.sum(g * g))
        c_i = float(clip_factors(np.array([n_i]), C)[0])
        for s, gl in zip(sums, grads):
            for dst, g in zip(s, gl):
                if isinstance(g, tuple):
                    rows, R = g
                    dst[rows] += c_i * R
                else:
                    dst += c_i * g
        sq[i] = n_i
        cs[i] = c_i
    return sums, sq, cs


# --------------------------------------------------------------------------------------
# Philox4x32-10 and the noise stream
# --------------------------------------------------------------------------------------

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = np.uint64(0x9E3779B9)
_W1 = np.uint64(0xBB67AE85)
_MASK = np.uint64(0xFFFFFFFF)
_S32 = np.uint64(32)


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Ten rounds of the Philox-4x32 bijection (Salmon, Moraes, Dror, Shaw, SC'11) on arrays of
    32-bit words held in uint64.  One round: the two products M0*c0 and M1*c2 are split into
    high and low halves; the new counter is (hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0); the key is
    advanced by the Weyl constants between rounds."""
    c0, c1, c2, c3 = (np.asarray(c, dtype=np.uint64) & _MASK for c in (c0, c1, c2, c3))
    k0 = np.uint64(k0) & _MASK
    k1 = np.uint64(k1) & _MASK
    for r in range(10):
        if r > 0:
            k0 = (k0 + _W0) & _MASK
            k1 = (k1 + _W1) & _MASK
        p0 = _M0 * c0
        p1 = _M1 * c2
        hi0, lo0 = p0 >> _S32, p0 & _MASK
        hi1, lo1 = p1 >> _S32, p1 & _MASK
        c0, c1, c2, c3 = (hi1 ^ c1 ^ k0), lo1, (hi0 ^ c3 ^ k1), lo0
    return c0, c1, c2, c3


def philox_u32(n: int, elem_offset: int, seed: int, step: int) -> np.ndarray:
    """Raw 32-bit words serving flat elements [elem_offset, elem_offset + n): element e takes word
    e mod 4 of the block with counter (lo32(e/4), hi32(e/4), lo32(step), hi32(step)) and key
    (lo32(seed), hi32(seed))."""
    if n == 0:
        return np.zeros(0, dtype=np.uint32)
    first = elem_offset // 4
    last = (elem_offset + n - 1) // 4
    j = np.arange(first, last + 1, dtype=np.uint64)
    w = philox4x32_10(j & _MASK, j >> _S32, np.uint64(step & 0xFFFFFFFF), np.uint64((step >> 32) & 0xFFFFFFFF),
                      seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    words = np.stack([x.astype(np.uint32) for x in w], axis=1).reshape(-1)
    s = elem_offset - 4 * first
    return words[s:s + n]


def uniform_from_u32(r: np.ndarray) -> np.ndarray:
    """u = ((r >> 9) + 1/2) / 2^23, in (0, 1); every value is exactly representable in fp32."""
    return ((np.asarray(r, dtype=np.uint32) >> np.uint32(9)).astype(np.float64) + 0.5) * (2.0 ** -23)


def normals(n: int, elem_offset: int, seed: int, step: int) -> np.ndarray:
    """Standard normals for flat elements [elem_offset, elem_offset + n).  Box-Muller on the word pairs
    (r0, r1) and (r2, r3) of each block: rho = sqrt(-2 ln u(r_even)), angle = 2 pi u(r_odd);
    the even element gets rho cos(angle), the odd one rho sin(angle)."""
    if n == 0:
        return np.zeros(0)
    first = (elem_offset // 4) * 4
    last = ((elem_offset + n + 3) // 4) * 4
    u = uniform_from_u32(philox_u32(last - first, first, seed, step)).reshape(-1, 2)
    rho = np.sqrt(-2.0 * np.log(u[:, 0]))
    ang = 2.0 * np.pi * u[:, 1]
    z = np.stack([rho * np.cos(ang), rho * np.sin(ang)], axis=1).reshape(-1)
    s = elem_offset - first
    return z[s:s + n]


# --------------------------------------------------------------------------------------
# noise + Adam with decoupled weight decay
# --------------------------------------------------------------------------------------


def noise_adamw(theta, m, v, S, *, elem_offset: int, sigma: float, C: float, seed: int, step: int,
                batch_size: int, lr: float, beta1: float, beta2: float, eps: float, weight_decay: float):
    """One update of a contiguous slice of the flat parameter space.  Returns fp64
    (theta, m, v, g).  Scalars are taken at the fp32 values the C ABI carries."""
    theta = to_f64(theta)
    m = to_f64(m)
    v = to_f64(v)
    S = to_f64(S)
    f = lambda x: float(np.float32(x))
    sigma, C, lr, beta1, beta2, eps, wd = map(f, (sigma, C, lr, beta1, beta2, eps, weight_decay))
    n = theta.shape[0]
    if sigma != 0.0:
        z = normals(n, elem_offset, seed, step)
        g = (S + sigma * C * z) / float(batch_size)
    else:
        g = S / float(batch_size)
    m_new = beta1 * m + (1.0 - beta1) * g
    v_new = beta2 * v + (1.0 - beta2) * g * g
    m_hat = m_new / (1.0 - beta1 ** step)
    v_hat = v_new / (1.0 - beta2 ** step)
    theta_new = theta - lr * (m_hat / (np.sqrt(v_hat) + eps) + wd * theta)
    return theta_new, m_new, v_new, g


# --------------------------------------------------------------------------------------
# gradient signal-to-noise ratio (the batch-size study of the experiments section)
# --------------------------------------------------------------------------------------


def gradient_snr_terms(S, *, elem_offset: int, sigma: float, C: float, seed: int, step: int):
    """Squared L2 norms of the two vectors whose ratio the paper tracks over training: the aggregated
    (clipped, summed) gradient S and the noise vector sigma*C*z that the update adds to it, over the
    flat elements [elem_offset, elem_offset + len(S)).  Both are taken before the division by |B_t|
    (which cancels in the ratio).  The noise vector is the one noise_adamw draws for the same
    (seed, step, element)."""
    S = to_f64(S)
    f = lambda x: float(np.float32(x))
    sigma, C = f(sigma), f(C)
    signal_sq = float(np.sum(S * S))
    if sigma == 0.0:
        return signal_sq, 0.0
    noise = sigma * C * normals(S.shape[0], elem_offset, seed, step)
    return signal_sq, float(np.sum(noise * noise))


def gradient_snr(signal_sq: float, noise_sq: float) -> float:
    """||S||_2 / ||sigma C z||_2 from the two squared norms (summed over slices by the caller)."""
    return float(np.sqrt(signal_sq / noise_sq)) if noise_sq > 0 else float("inf")


# --------------------------------------------------------------------------------------
# schedules (host-side scalars of Algorithm 1: the batch sizes q_t and the learning rates eta_t)
# --------------------------------------------------------------------------------------


def batch_size_schedule(step: int, b_start: int, b_end: int, ramp_steps: int, n_increments: int) -> int:
    """Increasing batch-size schedule of the batch-size study: the batch grows from b_start to b_end over
    ramp_steps steps, in n_increments equal jumps, one after every ramp_steps/n_increments completed steps
    (the paper: 262,144 -> 1,048,576 over 7,500 steps, a jump of 196,608 after each quarter, 1,048,576 from
    the end of the ramp on).  `step` counts from 1 as in Algorithm 1; step t has t - 1 completed steps
    before it.  Reading of what the text leaves open: jumps are equal, (b_end - b_start) / n_increments
    rounded down, with the last jump landing exactly on b_end."""
    if step < 1 or n_increments < 1 or ramp_steps < n_increments or b_end < b_start:
        raise ValueError("bad schedule arguments")
    done = step - 1
    k = min(n_increments, (done * n_increments) // ramp_steps)
    if k == n_increments:
        return b_end
    return b_start + k * ((b_end - b_start) // n_increments)


def lr_schedule(step: int, peak: float, warmup_steps: int, total_steps: int) -> float:
    """Linear warm-up to `peak` over warmup_steps steps, then quadratic decay to zero at total_steps
    (hyper-parameter tuning section: 7,500 warm-up steps of 20,000).  Reading of the unspecified form of the
    decay: eta_t = peak * ((total - t) / (total - warmup))^2 for t > warmup; eta_t = peak * t / warmup up to
    and including t = warmup; 0 beyond total_steps."""
    if step < 1 or warmup_steps < 0 or total_steps < max(1, warmup_steps):
        raise ValueError("bad schedule arguments")
    if step <= warmup_steps:
        return peak * step / warmup_steps
    if step >= total_steps:
        return 0.0
    frac = (total_steps - step) / (total_steps - warmup_steps)
    return peak * frac * frac


# --------------------------------------------------------------------------------------
# privacy accounting over a schedule of batch sizes (Renyi DP composition, Section 3)
# --------------------------------------------------------------------------------------


def rdp_sampled_gaussian(q: float, sigma: float, alpha: int) -> float:
    """Renyi divergence of integer order alpha >= 2 between one step's output distributions on neighbouring
    data sets: the Gaussian mechanism with noise multiplier sigma applied to a Poisson sample of rate q
    (Mironov, Talwar, Zhang, "Renyi differential privacy of the sampled Gaussian mechanism"):
        eps(alpha) = ln( sum_{k=0..alpha} C(alpha,k) (1-q)^(alpha-k) q^k exp((k^2 - k) / (2 sigma^2)) ) / (alpha - 1),
    written out term by term in 60-digit decimal arithmetic."""
    from decimal import Decimal, getcontext
    from math import comb

    if not (0.0 <= q <= 1.0) or sigma <= 0 or alpha < 2:
        raise ValueError("bad accounting arguments")
    from decimal import MAX_EMAX, MIN_EMIN

    ctx = getcontext()
    ctx.prec, ctx.Emax, ctx.Emin = 60, MAX_EMAX, MIN_EMIN   # exp((k^2-k)/(2 sigma^2)) leaves the default exponent range for small sigma
    qd, sd = Decimal(q), Decimal(sigma)
    total = Decimal(0)
    power = lambda x, n: Decimal(1) if n == 0 else x ** n   # 0^0 = 1 (the decimal module refuses it)
    for k in range(alpha + 1):
        total += Decimal(comb(alpha, k)) * power(1 - qd, alpha - k) * power(qd, k) * (Decimal(k * k - k) / (2 * sd * sd)).exp()
    return float(total.ln() / (alpha - 1))


def rdp_epsilon(q, steps, sigma: float, delta: float, max_alpha: int = 256):
    """(eps, best alpha) of a run made of phases: phase p takes steps[p] steps at sampling rate q[p] (batch size over
    data-set size), all with noise multiplier sigma.  By composition the run is (alpha, sum_p steps[p] * eps_p(alpha))-RDP
    for every alpha (the paper's accounting for the increasing batch-size schedule); the (eps, delta) guarantee is the
    best conversion over integer orders 2..max_alpha, eps = RDP(alpha) + ln(1/delta) / (alpha - 1) (Mironov,
    "Renyi differential privacy", Proposition 3).  Reading: the paper names the accountant but not the conversion."""
    import math

    if len(q) != len(steps) or not (0.0 < delta < 1.0) or max_alpha < 2:
        raise ValueError("bad accounting arguments")
    best = (float("inf"), 0)
    for alpha in range(2, max_alpha + 1):
        rdp = sum(n * rdp_sampled_gaussian(qq, sigma, alpha) for qq, n in zip(q, steps))
        eps = rdp + math.log(1.0 / delta) / (alpha - 1)
        if eps < best[0]:
            best = (eps, alpha)
    return best


def rdp_noise_multiplier(q, steps, eps_target: float, delta: float, max_alpha: int = 256, rel_tol: float = 1e-6) -> float:
    """The noise multiplier of Algorithm 1 for a privacy target (Section 3: the accountant is used to compute it):
    the smallest sigma, to a relative rel_tol, for which the run's guarantee as rdp_epsilon computes it is at most
    eps_target.  The guarantee shrinks as sigma grows, so: from sigma = 1, double until the target is met and halve
    until it is missed (a bracket lo < hi with eps(lo) > target >= eps(hi)), bisect until hi - lo <= rel_tol * hi, and
    return hi, the end that meets the target.  ValueError if even sigma = 2^20 misses it (the conversion term
    ln(1/delta) / (max_alpha - 1) alone is above the target)."""
    if not eps_target > 0.0 or not 0.0 < rel_tol < 1.0:
        raise ValueError("bad accounting arguments")
    eps_of = lambda sigma: rdp_epsilon(q, steps, sigma, delta, max_alpha)[0]
    hi = 1.0
    while eps_of(hi) > eps_target:
        hi *= 2.0
        if hi > 2.0 ** 20:
            raise ValueError("the target cannot be met with orders up to max_alpha")
    lo = hi / 2.0
    while eps_of(lo) <= eps_target:
        hi, lo = lo, lo / 2.0
        if lo < 2.0 ** -10:
            return hi   # no noise to speak of is needed (no steps, or nothing is ever sampled)
    while hi - lo > rel_tol * hi:
        mid = 0.5 * (lo + hi)
        if eps_of(mid) <= eps_target:
            hi = mid
        else:
            lo = mid
    return hi
