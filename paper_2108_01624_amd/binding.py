"""ctypes binding of libdpclip.so: one Python function per C entry point, same names, argument
marshalling only (tensor -> device pointer, dtype -> enum).  Every step of the path runs in the
library's HIP kernels; there is no fallback: if the library is missing, loading raises."""
from __future__ import annotations

import ctypes
import os
from ctypes import c_char_p, c_float, c_int, c_size_t, c_uint64, c_void_p

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libdpclip.so")
_lib = None

DP_F32, DP_BF16 = 0, 1
DP_PATH_AUTO, DP_PATH_GRAM, DP_PATH_MATERIALISE = 0, 1, 2
DP_PROF_WGEMM, DP_PROF_GRAM, DP_PROF_ADAMW = 0, 1, 2
DP_OK = 0
STATUS_NAMES = {0: "DP_OK", -1: "DP_ERR_NULL", -2: "DP_ERR_SHAPE", -3: "DP_ERR_DTYPE", -4: "DP_ERR_ALIGN",
                -5: "DP_ERR_VALUE", -6: "DP_ERR_INDEX", -7: "DP_ERR_WORKSPACE", -8: "DP_ERR_HIP"}

# name -> argument types (all return dp_status unless listed in _RESTYPES)
SIGNATURES = {
    "dp_create": [ctypes.POINTER(c_void_p), c_void_p, c_size_t],
    "dp_destroy": [c_void_p],
    "dp_sync": [c_void_p],
    "dp_status_str": [c_int],
    "dp_last_error": [c_void_p],
    "dp_sqnorms_dense": [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_int, c_int, c_int, c_void_p],
    "dp_sqnorms_dense_batched": [c_void_p, c_int, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_int, c_int, c_int, c_void_p],
    "dp_sqnorms_dense_shared": [c_void_p, c_int, c_void_p, c_int, c_void_p, c_int, c_int, c_int, c_int, c_int, c_int, c_void_p],
    "dp_sqnorms_layernorm": [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_void_p],
    "dp_sqnorms_embedding": [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_int, c_int, c_void_p],
    "dp_clip_factors": [c_void_p, c_void_p, c_int, c_float, c_void_p],
    "dp_clip_accumulate_dense": [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_int, c_float, c_void_p,
                                 c_void_p, c_void_p],
    "dp_clip_accumulate_dense_batched": [c_void_p, c_int, ctypes.POINTER(c_void_p), ctypes.POINTER(c_void_p), c_int, c_int,
                                         c_int, c_int, c_int, c_float, c_void_p, ctypes.POINTER(c_void_p),
                                         ctypes.POINTER(c_void_p)],
    "dp_clip_accumulate_layernorm": [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_float, c_void_p,
                                     c_void_p, c_void_p],
    "dp_clip_accumulate_embedding": [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_int, c_float, c_void_p,
                                     c_void_p],
    "dp_clip_accumulate_positions": [c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_float, c_void_p, c_void_p],
    "dp_sqnorms_layernorm_batched": [c_void_p, c_int, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_void_p],
    "dp_clip_accumulate_layernorm_batched": [c_void_p, c_int, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_float,
                                             c_void_p, c_void_p, c_void_p],
    "dp_sqnorms_layernorm_keep": [c_void_p, c_int, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_void_p, c_void_p],
    "dp_clip_accumulate_layernorm_kept": [c_void_p, c_int, c_void_p, c_int, c_int, c_float, c_void_p, c_void_p, c_void_p],
    "dp_sqnorms_tied_embedding": [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_int, c_int,
                                  c_void_p],
    "dp_clip_accumulate_tied_embedding": [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_int,
                                          c_int, c_float, c_void_p, c_void_p],
    "dp_noise_adamw": [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_uint64, c_uint64, c_float, c_float, c_uint64,
                       c_uint64, c_uint64, c_float, c_float, c_float, c_float, c_float, c_int],
    "dp_noise_adamw_snr": [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_uint64, c_uint64, c_float, c_float, c_uint64,
                           c_uint64, c_uint64, c_float, c_float, c_float, c_float, c_float, c_int, c_void_p],
    "dp_noise_adamw_snr_static": [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_uint64, c_uint64, c_float, c_float,
                                  c_uint64, c_uint64, c_uint64, c_float, c_float, c_float, c_float, c_float, c_int, c_void_p],
    "dp_zero_f32": [c_void_p, c_void_p, c_uint64],
    "dp_philox_u32": [c_void_p, c_void_p, c_uint64, c_uint64, c_uint64, c_uint64],
    "dp_normal_f32": [c_void_p, c_void_p, c_uint64, c_uint64, c_uint64, c_uint64],
    "dp_choose_path": [c_int, c_int, c_int, c_int, ctypes.POINTER(c_int)],
    "dp_gram_unit_plan": [c_int, ctypes.POINTER(ctypes.c_uint32), c_int, ctypes.POINTER(c_int)],
    "dp_batch_size_schedule": [c_uint64, c_uint64, c_uint64, c_uint64, ctypes.c_uint32, ctypes.POINTER(c_uint64)],
    "dp_lr_schedule": [c_uint64, ctypes.c_double, c_uint64, c_uint64, ctypes.POINTER(ctypes.c_double)],
    "dp_rdp_sampled_gaussian": [ctypes.c_double, ctypes.c_double, c_int, ctypes.POINTER(ctypes.c_double)],
    "dp_rdp_epsilon": [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(c_uint64), c_int, ctypes.c_double, ctypes.c_double,
                       c_int, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(c_int)],
    "dp_rdp_noise_multiplier": [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(c_uint64), c_int, ctypes.c_double, ctypes.c_double,
                                c_int, ctypes.c_double, ctypes.POINTER(ctypes.c_double)],
    "dp_profile_enable": [c_void_p, c_int],
    "dp_profile_read": [c_void_p, c_int, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(c_uint64),
                        ctypes.POINTER(ctypes.c_double)],
    "dp_profile_mfma_ceiling": [c_void_p, c_int, c_int, ctypes.POINTER(ctypes.c_double)],
}
_RESTYPES = {"dp_status_str": c_char_p, "dp_last_error": c_char_p}


class DpError(RuntimeError):
    def __init__(self, status: int, where: str, detail: str = ""):
        self.status = status
        super().__init__(f"{where}: {STATUS_NAMES.get(status, status)}" + (f" ({detail})" if detail else ""))


def load_library():
    """dlopen libdpclip.so and declare the prototypes.  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    # torch ships its own HIP runtime: import it first so that the library binds to the runtime that owns
    # the tensors' memory and streams instead of pulling in a second copy.
    import torch  # noqa: F401

    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python -m paper_2108_01624_amd.build` "
                           "(there is no fallback path)")
    lib = ctypes.CDLL(_LIB_PATH)
    for name, argtypes in SIGNATURES.items():
        fn = getattr(lib, name)
        fn.argtypes = argtypes
        fn.restype = _RESTYPES.get(name, c_int)
    _lib = lib
    return lib


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _f32(t):
    """Device pointer of an fp32 tensor (sums, norms, parameters); refuses any other element type."""
    if t is None or isinstance(t, int):
        return t
    import torch

    if t.dtype != torch.float32:
        raise TypeError(f"expected a float32 tensor, got {t.dtype}")
    return t.data_ptr()


def _i32(t):
    if t is None or isinstance(t, int):
        return t
    import torch

    if t.dtype != torch.int32:
        raise TypeError(f"expected an int32 tensor, got {t.dtype}")
    return t.data_ptr()


def _dtype_of(t) -> int:
    import torch

    if t.dtype == torch.float32:
        return DP_F32
    if t.dtype == torch.bfloat16:
        return DP_BF16
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def _check(ctx, st: int, where: str):
    if st != DP_OK:
        detail = load_library().dp_last_error(ctx).decode() if ctx else ""
        raise DpError(st, where, detail)


# ---- one function per entry point (same names as the C ABI) ---------------------------------------
def dp_create(stream_handle: int = 0, workspace_bytes: int = 0) -> int:
    h = c_void_p()
    st = load_library().dp_create(ctypes.byref(h), c_void_p(stream_handle), workspace_bytes)
    if st != DP_OK:
        raise DpError(st, "dp_create")
    return h.value


def dp_destroy(ctx):
    _check(None, load_library().dp_destroy(ctx), "dp_destroy")


def dp_sync(ctx):
    _check(ctx, load_library().dp_sync(ctx), "dp_sync")


def dp_status_str(s: int) -> str:
    return load_library().dp_status_str(s).decode()


def dp_last_error(ctx) -> str:
    return load_library().dp_last_error(ctx).decode()


def dp_sqnorms_dense(ctx, A, G, has_bias, path, sqnorms, *, B=None, T=None):
    B = A.shape[0] if B is None else B
    T = A.shape[1] if T is None else T
    st = load_library().dp_sqnorms_dense(ctx, _ptr(A), _ptr(G), _dtype_of(A), B, T, A.shape[-1], G.shape[-1],
                                         int(has_bias), int(path), _f32(sqnorms))
    _check(ctx, st, "dp_sqnorms_dense")


def dp_sqnorms_dense_batched(ctx, As, Gs, has_bias, path, sqnorms):
    """As, Gs: equally long lists of same-shaped tensors (one pair per layer)."""
    n = len(As)
    B, T, d_in = As[0].shape
    d_out = Gs[0].shape[-1]
    for a, g in zip(As, Gs):
        if tuple(a.shape) != (B, T, d_in) or tuple(g.shape) != (B, T, d_out) or a.dtype != As[0].dtype:
            raise ValueError("all layers of a batch must share one shape and dtype")
    arr = lambda ptrs: (c_void_p * n)(*ptrs)
    st = load_library().dp_sqnorms_dense_batched(ctx, n, arr([_ptr(t) for t in As]), arr([_ptr(t) for t in Gs]),
                                                 _dtype_of(As[0]), B, T, d_in, d_out, int(has_bias), int(path), _f32(sqnorms))
    _check(ctx, st, "dp_sqnorms_dense_batched")


def dp_sqnorms_dense_shared(ctx, As, Gs, has_bias, sqnorms):
    """As: one input tensor per group; Gs: per group a list of the output-gradient tensors of the layers sharing it."""
    ng, n_out = len(As), len(Gs[0])
    B, T, d_in = As[0].shape
    d_out = Gs[0][0].shape[-1]
    flat = []
    for a, gs in zip(As, Gs):
        if tuple(a.shape) != (B, T, d_in) or len(gs) != n_out or a.dtype != As[0].dtype:
            raise ValueError("all groups must share one shape, dtype and layer count")
        for g in gs:
            if tuple(g.shape) != (B, T, d_out) or g.dtype != a.dtype:
                raise ValueError("all layers of a call must share one shape and dtype")
            flat.append(g)
    pa = (c_void_p * ng)(*[_ptr(t) for t in As])
    pg = (c_void_p * len(flat))(*[_ptr(t) for t in flat])
    st = load_library().dp_sqnorms_dense_shared(ctx, ng, pa, n_out, pg, _dtype_of(As[0]), B, T, d_in, d_out, int(has_bias),
                                                _f32(sqnorms))
    _check(ctx, st, "dp_sqnorms_dense_shared")


def dp_sqnorms_layernorm(ctx, Xhat, G, sqnorms):
    B, T, d = Xhat.shape
    _check(ctx, load_library().dp_sqnorms_layernorm(ctx, _ptr(Xhat), _ptr(G), _dtype_of(G), B, T, d, _f32(sqnorms)),
           "dp_sqnorms_layernorm")


def dp_sqnorms_embedding(ctx, ids, G, V, distinct_per_example, sqnorms):
    B, T, d = G.shape
    st = load_library().dp_sqnorms_embedding(ctx, _i32(ids), _ptr(G), _dtype_of(G), B, T, d, int(V),
                                             int(distinct_per_example), _f32(sqnorms))
    _check(ctx, st, "dp_sqnorms_embedding")


def dp_clip_factors(ctx, sqnorms, C, c):
    _check(ctx, load_library().dp_clip_factors(ctx, _f32(sqnorms), sqnorms.shape[0], float(C), _f32(c)), "dp_clip_factors")


def dp_clip_accumulate_dense(ctx, A, G, C, sqnorms, sum_W, sum_b=None):
    B, T, d_in = A.shape
    st = load_library().dp_clip_accumulate_dense(ctx, _ptr(A), _ptr(G), _dtype_of(A), B, T, d_in, G.shape[-1], float(C),
                                                 _f32(sqnorms), _f32(sum_W), _f32(sum_b))
    _check(ctx, st, "dp_clip_accumulate_dense")


def dp_clip_accumulate_dense_batched(ctx, As, Gs, C, sqnorms, sum_Ws, sum_bs=None):
    """As, Gs, sum_Ws (and sum_bs, entries may be None): equally long lists of same-shaped tensors."""
    n = len(As)
    B, T, d_in = As[0].shape
    d_out = Gs[0].shape[-1]
    for a, g in zip(As, Gs):
        if tuple(a.shape) != (B, T, d_in) or tuple(g.shape) != (B, T, d_out) or a.dtype != As[0].dtype:
            raise ValueError("all layers of a batch must share one shape and dtype")
    arr = lambda ptrs: (c_void_p * n)(*ptrs)
    pb = arr([_f32(t) for t in sum_bs]) if sum_bs is not None else None
    st = load_library().dp_clip_accumulate_dense_batched(ctx, n, arr([_ptr(t) for t in As]), arr([_ptr(t) for t in Gs]),
                                                         _dtype_of(As[0]), B, T, d_in, d_out, float(C), _f32(sqnorms),
                                                         arr([_f32(t) for t in sum_Ws]), pb)
    _check(ctx, st, "dp_clip_accumulate_dense_batched")


def dp_clip_accumulate_layernorm(ctx, Xhat, G, C, sqnorms, sum_gamma, sum_beta):
    B, T, d = Xhat.shape
    st = load_library().dp_clip_accumulate_layernorm(ctx, _ptr(Xhat), _ptr(G), _dtype_of(G), B, T, d, float(C),
                                                     _f32(sqnorms), _f32(sum_gamma), _f32(sum_beta))
    _check(ctx, st, "dp_clip_accumulate_layernorm")


def dp_clip_accumulate_embedding(ctx, ids, G, V, C, sqnorms, sum_E):
    B, T, d = G.shape
    st = load_library().dp_clip_accumulate_embedding(ctx, _i32(ids), _ptr(G), _dtype_of(G), B, T, d, int(V), float(C),
                                                     _f32(sqnorms), _f32(sum_E))
    _check(ctx, st, "dp_clip_accumulate_embedding")


def dp_clip_accumulate_positions(ctx, G, C, sqnorms, sum_E):
    B, T, d = G.shape
    if sum_E.numel() < T * d:
        raise ValueError("sum_E must hold at least T rows")
    st = load_library().dp_clip_accumulate_positions(ctx, _ptr(G), _dtype_of(G), B, T, d, float(C), _f32(sqnorms), _f32(sum_E))
    _check(ctx, st, "dp_clip_accumulate_positions")


def _same_shaped(Xs, Gs):
    shp, dt = tuple(Xs[0].shape), Xs[0].dtype
    for x, g in zip(Xs, Gs):
        if tuple(x.shape) != shp or tuple(g.shape) != shp or x.dtype != dt or g.dtype != dt:
            raise ValueError("all layers of a batch must share one shape and dtype")
    return shp


def dp_sqnorms_layernorm_batched(ctx, Xhats, Gs, sqnorms):
    """Xhats, Gs: equally long lists of same-shaped tensors."""
    n = len(Xhats)
    B, T, d = _same_shaped(Xhats, Gs)
    arr = lambda ptrs: (c_void_p * n)(*ptrs)
    st = load_library().dp_sqnorms_layernorm_batched(ctx, n, arr([_ptr(t) for t in Xhats]), arr([_ptr(t) for t in Gs]),
                                                     _dtype_of(Gs[0]), B, T, d, _f32(sqnorms))
    _check(ctx, st, "dp_sqnorms_layernorm_batched")


def dp_clip_accumulate_layernorm_batched(ctx, Xhats, Gs, C, sqnorms, sum_gammas, sum_betas):
    n = len(Xhats)
    B, T, d = _same_shaped(Xhats, Gs)
    arr = lambda ptrs: (c_void_p * n)(*ptrs)
    st = load_library().dp_clip_accumulate_layernorm_batched(
        ctx, n, arr([_ptr(t) for t in Xhats]), arr([_ptr(t) for t in Gs]), _dtype_of(Gs[0]), B, T, d, float(C), _f32(sqnorms),
        arr([_f32(t) for t in sum_gammas]), arr([_f32(t) for t in sum_betas]))
    _check(ctx, st, "dp_clip_accumulate_layernorm_batched")


def dp_sqnorms_layernorm_keep(ctx, Xhats, Gs, sqnorms, grads):
    """grads: one float32 tensor [B, 2, d] per layer, overwritten with every example's gain / offset gradient."""
    n = len(Xhats)
    B, T, d = _same_shaped(Xhats, Gs)
    for g in grads:
        if g.numel() < B * 2 * d:
            raise ValueError("grads[l] must hold B x 2 x d floats")
    arr = lambda ptrs: (c_void_p * n)(*ptrs)
    st = load_library().dp_sqnorms_layernorm_keep(ctx, n, arr([_ptr(t) for t in Xhats]), arr([_ptr(t) for t in Gs]),
                                                  _dtype_of(Gs[0]), B, T, d, _f32(sqnorms), arr([_f32(t) for t in grads]))
    _check(ctx, st, "dp_sqnorms_layernorm_keep")


def dp_clip_accumulate_layernorm_kept(ctx, grads, B, d, C, sqnorms, sum_gammas, sum_betas):
    n = len(grads)
    arr = lambda ptrs: (c_void_p * n)(*ptrs)
    st = load_library().dp_clip_accumulate_layernorm_kept(ctx, n, arr([_f32(t) for t in grads]), int(B), int(d), float(C),
                                                          _f32(sqnorms), arr([_f32(t) for t in sum_gammas]),
                                                          arr([_f32(t) for t in sum_betas]))
    _check(ctx, st, "dp_clip_accumulate_layernorm_kept")


def _tied_shapes(ids, dY, H, dL):
    B, T, d = dY.shape
    M, V = dL.shape[1], dL.shape[2]
    if tuple(ids.shape) != (B, T) or tuple(H.shape) != (B, M, d) or dL.shape[0] != B:
        raise ValueError("ids [B,T], dY [B,T,d], H [B,M,d], dL [B,M,V] expected")
    if H.dtype != dY.dtype or dL.dtype != dY.dtype:
        raise ValueError("dY, H and dL must share one dtype")
    return B, T, M, d, V


def dp_sqnorms_tied_embedding(ctx, ids, dY, H, dL, sqnorms):
    B, T, M, d, V = _tied_shapes(ids, dY, H, dL)
    st = load_library().dp_sqnorms_tied_embedding(ctx, _i32(ids), _ptr(dY), _ptr(H), _ptr(dL), _dtype_of(dY), B, T, M, d, V,
                                                  _f32(sqnorms))
    _check(ctx, st, "dp_sqnorms_tied_embedding")


def dp_clip_accumulate_tied_embedding(ctx, ids, dY, H, dL, C, sqnorms, sum_E):
    B, T, M, d, V = _tied_shapes(ids, dY, H, dL)
    if sum_E.numel() != V * d:
        raise ValueError("sum_E must be [V, d]")
    st = load_library().dp_clip_accumulate_tied_embedding(ctx, _i32(ids), _ptr(dY), _ptr(H), _ptr(dL), _dtype_of(dY), B, T, M,
                                                          d, V, float(C), _f32(sqnorms), _f32(sum_E))
    _check(ctx, st, "dp_clip_accumulate_tied_embedding")


def dp_noise_adamw(ctx, params, m, v, sum_, *, n=None, elem_offset=0, sigma, C, seed, step, batch_size, lr, beta1, beta2,
                   eps=1e-11, weight_decay, zero_sum=False):
    n = params.numel() if n is None else n
    st = load_library().dp_noise_adamw(ctx, _f32(params), _f32(m), _f32(v), _f32(sum_), n, elem_offset, sigma, C, seed,
                                       step, batch_size, lr, beta1, beta2, eps, weight_decay, int(zero_sum))
    _check(ctx, st, "dp_noise_adamw")


def dp_noise_adamw_snr(ctx, params, m, v, sum_, snr_sq, *, n=None, elem_offset=0, sigma, C, seed, step, batch_size, lr,
                       beta1, beta2, eps=1e-11, weight_decay, zero_sum=False):
    n = params.numel() if n is None else n
    if snr_sq.numel() < 2:
        raise ValueError("snr_sq needs two floats")
    st = load_library().dp_noise_adamw_snr(ctx, _f32(params), _f32(m), _f32(v), _f32(sum_), n, elem_offset, sigma, C,
                                           seed, step, batch_size, lr, beta1, beta2, eps, weight_decay, int(zero_sum),
                                           _f32(snr_sq))
    _check(ctx, st, "dp_noise_adamw_snr")


def dp_noise_adamw_snr_static(stream_handle, params, m, v, sum_, snr_sq, *, n=None, elem_offset=0, sigma, C, seed, step,
                              batch_size, lr, beta1, beta2, eps=1e-11, weight_decay, zero_sum=False):
    """dp_noise_adamw_snr without a context: `stream_handle` is the hipStream_t as an integer (0 = the null stream)."""
    n = params.numel() if n is None else n
    if snr_sq.numel() < 2:
        raise ValueError("snr_sq needs two floats")
    st = load_library().dp_noise_adamw_snr_static(stream_handle, _f32(params), _f32(m), _f32(v), _f32(sum_), n, elem_offset,
                                                  sigma, C, seed, step, batch_size, lr, beta1, beta2, eps, weight_decay,
                                                  int(zero_sum), _f32(snr_sq))
    if st != DP_OK:
        raise DpError(st, "dp_noise_adamw_snr_static")


def dp_zero_f32(ctx, p, n=None):
    _check(ctx, load_library().dp_zero_f32(ctx, _f32(p), p.numel() if n is None else n), "dp_zero_f32")


def dp_philox_u32(ctx, out, elem_offset, seed, step, n=None):
    _check(ctx, load_library().dp_philox_u32(ctx, _i32(out), out.numel() if n is None else n, elem_offset, seed, step),
           "dp_philox_u32")


def dp_normal_f32(ctx, out, elem_offset, seed, step, n=None):
    _check(ctx, load_library().dp_normal_f32(ctx, _f32(out), out.numel() if n is None else n, elem_offset, seed, step),
           "dp_normal_f32")


def dp_batch_size_schedule(step, b_start, b_end, ramp_steps, n_increments) -> int:
    out = c_uint64()
    st = load_library().dp_batch_size_schedule(step, b_start, b_end, ramp_steps, n_increments, ctypes.byref(out))
    if st != DP_OK:
        raise DpError(st, "dp_batch_size_schedule")
    return out.value


def dp_lr_schedule(step, peak, warmup_steps, total_steps) -> float:
    out = ctypes.c_double()
    st = load_library().dp_lr_schedule(step, peak, warmup_steps, total_steps, ctypes.byref(out))
    if st != DP_OK:
        raise DpError(st, "dp_lr_schedule")
    return out.value


def dp_rdp_sampled_gaussian(q, sigma, alpha) -> float:
    out = ctypes.c_double()
    st = load_library().dp_rdp_sampled_gaussian(q, sigma, alpha, ctypes.byref(out))
    if st != DP_OK:
        raise DpError(st, "dp_rdp_sampled_gaussian")
    return out.value


def dp_rdp_epsilon(q, steps, sigma, delta, max_alpha=256):
    """(eps, best order) of a run of len(q) phases: steps[p] steps at sampling rate q[p]."""
    n = len(q)
    if len(steps) != n:
        raise ValueError("q and steps must be equally long")
    eps, arg = ctypes.c_double(), c_int()
    st = load_library().dp_rdp_epsilon((ctypes.c_double * n)(*q), (c_uint64 * n)(*steps), n, sigma, delta, max_alpha,
                                       ctypes.byref(eps), ctypes.byref(arg))
    if st != DP_OK:
        raise DpError(st, "dp_rdp_epsilon")
    return eps.value, arg.value


def dp_rdp_noise_multiplier(q, steps, eps_target, delta, max_alpha=256, rel_tol=1e-6) -> float:
    """Smallest noise multiplier (to rel_tol) whose (eps, delta) guarantee over the run is at most eps_target."""
    n = len(q)
    if len(steps) != n:
        raise ValueError("q and steps must be equally long")
    out = ctypes.c_double()
    st = load_library().dp_rdp_noise_multiplier((ctypes.c_double * n)(*q), (c_uint64 * n)(*steps), n, eps_target, delta,
                                                max_alpha, rel_tol, ctypes.byref(out))
    if st != DP_OK:
        raise DpError(st, "dp_rdp_noise_multiplier")
    return out.value


def dp_choose_path(T, d_in, d_out, dtype=DP_BF16) -> int:
    out = c_int()
    st = load_library().dp_choose_path(T, d_in, d_out, dtype, ctypes.byref(out))
    if st != DP_OK:
        raise DpError(st, "dp_choose_path")
    return out.value


def dp_gram_unit_plan(T) -> list:
    """The unit words of dp_gram_unit_plan for sequence length T (host only)."""
    buf = (ctypes.c_uint32 * 70)()
    n = c_int()
    st = load_library().dp_gram_unit_plan(T, buf, 70, ctypes.byref(n))
    if st != DP_OK:
        raise DpError(st, "dp_gram_unit_plan")
    return [int(buf[k]) for k in range(n.value)]


def dp_profile_enable(ctx, enable: bool):
    _check(ctx, load_library().dp_profile_enable(ctx, int(enable)), "dp_profile_enable")


def dp_profile_read(ctx, kind: int):
    """-> (milliseconds, launches, work) summed over the launches of `kind` since the last read."""
    ms, cnt, work = ctypes.c_double(), c_uint64(), ctypes.c_double()
    st = load_library().dp_profile_read(ctx, kind, ctypes.byref(ms), ctypes.byref(cnt), ctypes.byref(work))
    _check(ctx, st, "dp_profile_read")
    return ms.value, cnt.value, work.value


def dp_profile_mfma_ceiling(ctx, iters: int = 4096, launches: int = 8) -> float:
    """-> TFLOP/s that a register-only loop of the GEMM's bf16 matrix instructions sustains on this card."""
    out = ctypes.c_double()
    _check(ctx, load_library().dp_profile_mfma_ceiling(ctx, iters, launches, ctypes.byref(out)), "dp_profile_mfma_ceiling")
    return out.value


class Context:
    """A dp_ctx bound to torch's current HIP stream on the current device."""

    def __init__(self, workspace_bytes: int = 0, stream=None):
        import torch

        if not torch.cuda.is_available():
            raise RuntimeError("paper_2108_01624_amd needs a GPU: there is no CPU path")
        s = torch.cuda.current_stream() if stream is None else stream
        self.stream = s
        self.handle = dp_create(s.cuda_stream, workspace_bytes)

    def close(self):
        if self.handle:
            dp_destroy(self.handle)
            self.handle = None

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    def __getattr__(self, name):
        # ctx.sqnorms_dense(...) == dp_sqnorms_dense(ctx.handle, ...)
        fn = globals().get("dp_" + name)
        if fn is None:
            raise AttributeError(name)
        return lambda *a, **k: fn(self.handle, *a, **k)
