// C ABI entry points: argument checks, context management and dispatch to the kernel launchers.
#include <limits.h>
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include "dp_common.h"

namespace {

constexpr size_t DEFAULT_WORKSPACE = (size_t)512 << 20;
constexpr int CBUF_CAP = 1 << 20;

#define REQUIRE_CTX(ctx) \
    if (!(ctx)) return DP_ERR_NULL

#define FAIL(ctx, code, ...)          \
    do {                              \
        DP_SET_ERR(ctx, __VA_ARGS__); \
        return code;                  \
    } while (0)

dp_status check_dtype(dp_ctx* ctx, dp_dtype dt) {
    if (dt != DP_F32 && dt != DP_BF16) FAIL(ctx, DP_ERR_DTYPE, "unknown dtype %d", (int)dt);
    return DP_OK;
}

dp_status check_tensor(dp_ctx* ctx, const char* name, const void* p, dp_dtype dt, int width) {
    if (!p) FAIL(ctx, DP_ERR_NULL, "%s is NULL", name);
    if (dt == DP_BF16) {
        if (width % 8) FAIL(ctx, DP_ERR_SHAPE, "%s: width %d is not a multiple of 8 (bf16)", name, width);
        if ((uintptr_t)p & 15) FAIL(ctx, DP_ERR_ALIGN, "%s is not 16-byte aligned (bf16)", name);
    } else if ((uintptr_t)p & 3) {
        FAIL(ctx, DP_ERR_ALIGN, "%s is not 4-byte aligned", name);
    }
    return DP_OK;
}

dp_status check_f32(dp_ctx* ctx, const char* name, const void* p) {
    if (!p) FAIL(ctx, DP_ERR_NULL, "%s is NULL", name);
    if ((uintptr_t)p & 3) FAIL(ctx, DP_ERR_ALIGN, "%s is not 4-byte aligned", name);
    return DP_OK;
}

dp_status check_bt(dp_ctx* ctx, int B, int T) {
    if (B < 0 || T < 0) FAIL(ctx, DP_ERR_SHAPE, "negative B or T");
    if ((long)B * T > (long)INT_MAX - 4096) FAIL(ctx, DP_ERR_SHAPE, "B*T = %ld exceeds 2^31", (long)B * T);
    return DP_OK;
}

dp_status check_clip(dp_ctx* ctx, float C, int B) {
    if (!(C > 0.f) || !isfinite(C)) FAIL(ctx, DP_ERR_VALUE, "clip norm C must be positive and finite");
    if (B > ctx->cbuf_cap) FAIL(ctx, DP_ERR_WORKSPACE, "B = %d exceeds the clip-factor buffer (%d)", B, ctx->cbuf_cap);
    return DP_OK;
}

#define TRY(expr)                    \
    do {                             \
        dp_status s__ = (expr);      \
        if (s__ != DP_OK) return s__; \
    } while (0)

}  // namespace

extern "C" {

dp_status dp_create(dp_ctx** out, void* hip_stream, size_t workspace_bytes) {
    if (!out) return DP_ERR_NULL;
    dp_ctx* ctx = (dp_ctx*)calloc(1, sizeof(dp_ctx));
    if (!ctx) return DP_ERR_HIP;
    ctx->stream = (hipStream_t)hip_stream;
    ctx->ws_bytes = workspace_bytes ? workspace_bytes : DEFAULT_WORKSPACE;
    ctx->cbuf_cap = CBUF_CAP;
    ctx->prof = (dp_prof_rec*)calloc(DP_PROF_CAP, sizeof(dp_prof_rec));
    if (!ctx->prof) {
        free(ctx);
        return DP_ERR_HIP;
    }
    hipError_t e = hipGetDevice(&ctx->device);
    float* static_scratch = nullptr;  // looked up here so that dp_noise_adamw_snr_static finds it ready on this device
    if (e == hipSuccess && dpk_static_scratch(&static_scratch) != DP_OK) e = hipErrorInvalidSymbol;
    if (e == hipSuccess) e = hipMalloc((void**)&ctx->ws, ctx->ws_bytes);
    if (e == hipSuccess) e = hipMalloc((void**)&ctx->err_word, sizeof(int));
    if (e == hipSuccess) e = hipMalloc((void**)&ctx->cbuf, (size_t)ctx->cbuf_cap * sizeof(float));
    if (e == hipSuccess) e = hipMemset(ctx->err_word, 0, sizeof(int));
    if (e != hipSuccess) {
        if (ctx->ws) (void)hipFree(ctx->ws);
        if (ctx->err_word) (void)hipFree(ctx->err_word);
        if (ctx->cbuf) (void)hipFree(ctx->cbuf);
        free(ctx->prof);
        free(ctx);
        return DP_ERR_HIP;
    }
    *out = ctx;
    return DP_OK;
}

dp_status dp_destroy(dp_ctx* ctx) {
    REQUIRE_CTX(ctx);
    (void)hipStreamSynchronize(ctx->stream);
    (void)hipFree(ctx->ws);
    (void)hipFree(ctx->err_word);
    (void)hipFree(ctx->cbuf);
    for (int i = 0; i < ctx->prof_made; ++i) {
        (void)hipEventDestroy(ctx->prof[i].start);
        (void)hipEventDestroy(ctx->prof[i].stop);
    }
    free(ctx->prof);
    free(ctx);
    return DP_OK;
}

dp_status dp_profile_enable(dp_ctx* ctx, int enable) {
    REQUIRE_CTX(ctx);
    DP_HIP_CHECK(ctx, hipStreamSynchronize(ctx->stream));
    ctx->prof_on = enable ? 1 : 0;
    ctx->prof_n = 0;
    return DP_OK;
}

dp_status dp_profile_read(dp_ctx* ctx, dp_prof_kind kind, double* ms_total, uint64_t* launches, double* work_total) {
    REQUIRE_CTX(ctx);
    if ((int)kind < 0 || (int)kind > (int)DP_PROF_ADAMW) FAIL(ctx, DP_ERR_DTYPE, "unknown profile kind %d", (int)kind);
    DP_HIP_CHECK(ctx, hipStreamSynchronize(ctx->stream));
    double ms = 0.0, work = 0.0;
    uint64_t cnt = 0;
    int keep = 0;
    for (int i = 0; i < ctx->prof_n; ++i) {
        dp_prof_rec r = ctx->prof[i];
        if (r.kind == (int)kind) {
            float t = 0.f;
            DP_HIP_CHECK(ctx, hipEventElapsedTime(&t, r.start, r.stop));
            ms += t;
            work += r.work;
            ++cnt;
        }
    }
    // compact: drop the records just read, keep the others (event objects are swapped, never leaked)
    for (int i = 0; i < ctx->prof_n; ++i) {
        if (ctx->prof[i].kind != (int)kind) {
            if (i != keep) {
                dp_prof_rec t = ctx->prof[keep];
                ctx->prof[keep] = ctx->prof[i];
                ctx->prof[i] = t;
            }
            ++keep;
        }
    }
    ctx->prof_n = keep;
    if (ms_total) *ms_total = ms;
    if (launches) *launches = cnt;
    if (work_total) *work_total = work;
    return DP_OK;
}

dp_status dp_profile_mfma_ceiling(dp_ctx* ctx, int iters, int launches, double* tflops) {
    REQUIRE_CTX(ctx);
    if (!tflops) FAIL(ctx, DP_ERR_NULL, "tflops is NULL");
    if (iters < 1 || iters > (1 << 20) || launches < 1 || launches > 1024) FAIL(ctx, DP_ERR_VALUE, "iters in [1, 2^20], launches in [1, 1024]");
    return dpk_mfma_ceiling(ctx, iters, launches, tflops);
}

dp_status dp_sync(dp_ctx* ctx) {
    REQUIRE_CTX(ctx);
    DP_HIP_CHECK(ctx, hipStreamSynchronize(ctx->stream));
    int w = 0;
    DP_HIP_CHECK(ctx, hipMemcpy(&w, ctx->err_word, sizeof(int), hipMemcpyDeviceToHost));
    if (w) {
        DP_HIP_CHECK(ctx, hipMemset(ctx->err_word, 0, sizeof(int)));
        if (w & DP_ERRBIT_INDEX) FAIL(ctx, DP_ERR_INDEX, "a token id outside [0, V) was met on the device");
        FAIL(ctx, DP_ERR_VALUE, "a per-example squared norm was NaN or overflowed fp32: the sums it entered hold NaN");
    }
    return DP_OK;
}

const char* dp_status_str(dp_status s) {
    switch (s) {
        case DP_OK: return "DP_OK";
        case DP_ERR_NULL: return "DP_ERR_NULL";
        case DP_ERR_SHAPE: return "DP_ERR_SHAPE";
        case DP_ERR_DTYPE: return "DP_ERR_DTYPE";
        case DP_ERR_ALIGN: return "DP_ERR_ALIGN";
        case DP_ERR_VALUE: return "DP_ERR_VALUE";
        case DP_ERR_INDEX: return "DP_ERR_INDEX";
        case DP_ERR_WORKSPACE: return "DP_ERR_WORKSPACE";
        case DP_ERR_HIP: return "DP_ERR_HIP";
    }
    return "DP_ERR_UNKNOWN";
}

const char* dp_last_error(const dp_ctx* ctx) { return ctx ? ctx->msg : "no context"; }

dp_status dp_gram_unit_plan(int T, uint32_t* units, int capacity, int* n_units) {
    if (!units || !n_units) return DP_ERR_NULL;
    if (capacity < 0) return DP_ERR_SHAPE;
    return dpk_gram_unit_plan(T, units, capacity, n_units);
}

dp_status dp_choose_path(int T, int d_in, int d_out, dp_dtype dtype, dp_path* out) {
    if (!out) return DP_ERR_NULL;
    if (dtype != DP_F32 && dtype != DP_BF16) return DP_ERR_DTYPE;
    if (T < 0 || d_in < 0 || d_out < 0) return DP_ERR_SHAPE;
    // flops of the symmetric Gram form, T(T+1)/2 * (d_in + d_out) multiply-adds per example, against those
    // of materialising the d_in x d_out gradient, T * d_in * d_out.
    const double gram = 0.5 * ((double)T + 1.0) * ((double)d_in + (double)d_out);
    const double mat = (double)d_in * (double)d_out;
    *out = gram <= mat ? DP_PATH_GRAM : DP_PATH_MATERIALISE;
    return DP_OK;
}

dp_status dp_batch_size_schedule(uint64_t step, uint64_t b_start, uint64_t b_end, uint64_t ramp_steps,
                                 uint32_t n_increments, uint64_t* out) {
    if (!out) return DP_ERR_NULL;
    if (step == 0 || n_increments == 0 || ramp_steps < n_increments || b_end < b_start) return DP_ERR_VALUE;
    // k jumps have happened once k/n_increments of the ramp's steps are complete (step t has t - 1 behind it)
    const unsigned __int128 done = (unsigned __int128)(step - 1) * n_increments;
    const uint64_t k = (uint64_t)(done / ramp_steps);
    *out = k >= n_increments ? b_end : b_start + k * ((b_end - b_start) / n_increments);
    return DP_OK;
}

dp_status dp_lr_schedule(uint64_t step, double peak, uint64_t warmup_steps, uint64_t total_steps, double* out) {
    if (!out) return DP_ERR_NULL;
    if (step == 0 || total_steps == 0 || total_steps < warmup_steps || !isfinite(peak)) return DP_ERR_VALUE;
    if (step <= warmup_steps) {
        *out = peak * (double)step / (double)warmup_steps;
    } else if (step >= total_steps) {
        *out = 0.0;
    } else {
        const double frac = (double)(total_steps - step) / (double)(total_steps - warmup_steps);
        *out = peak * frac * frac;
    }
    return DP_OK;
}

// ln of one term of the sampled-Gaussian moment sum; -inf for a vanishing factor
static double rdp_log_term(double q, double sigma, int alpha, int k) {
    const double lq = q > 0.0 ? log(q) : -INFINITY, l1q = q < 1.0 ? log1p(-q) : -INFINITY;
    double t = lgamma(alpha + 1.0) - lgamma(k + 1.0) - lgamma(alpha - k + 1.0);
    if (k > 0) t += k * lq;
    if (alpha - k > 0) t += (alpha - k) * l1q;
    return t + ((double)k * k - k) / (2.0 * sigma * sigma);
}

dp_status dp_rdp_sampled_gaussian(double q, double sigma, int alpha, double* out) {
    if (!out) return DP_ERR_NULL;
    if (!(q >= 0.0 && q <= 1.0) || !(sigma > 0.0) || !isfinite(sigma) || alpha < 2) return DP_ERR_VALUE;
    // log-sum-exp over the alpha + 1 terms
    double mx = -INFINITY;
    for (int k = 0; k <= alpha; ++k) mx = fmax(mx, rdp_log_term(q, sigma, alpha, k));
    double acc = 0.0;
    for (int k = 0; k <= alpha; ++k) acc += exp(rdp_log_term(q, sigma, alpha, k) - mx);
    *out = (mx + log(acc)) / (alpha - 1.0);
    return DP_OK;
}

dp_status dp_rdp_epsilon(const double* q, const uint64_t* steps, int n_phases, double sigma, double delta, int max_alpha,
                         double* eps, int* best_alpha) {
    if (!q || !steps || !eps) return DP_ERR_NULL;
    if (n_phases < 0 || !(delta > 0.0 && delta < 1.0) || max_alpha < 2) return DP_ERR_VALUE;
    double best = INFINITY;
    int arg = 0;
    for (int alpha = 2; alpha <= max_alpha; ++alpha) {
        double rdp = 0.0;
        for (int p = 0; p < n_phases; ++p) {
            double e;
            const dp_status st = dp_rdp_sampled_gaussian(q[p], sigma, alpha, &e);
            if (st != DP_OK) return st;
            rdp += (double)steps[p] * e;
        }
        const double cand = rdp + log(1.0 / delta) / (alpha - 1.0);
        if (cand < best) {
            best = cand;
            arg = alpha;
        }
    }
    *eps = best;
    if (best_alpha) *best_alpha = arg;
    return DP_OK;
}

dp_status dp_rdp_noise_multiplier(const double* q, const uint64_t* steps, int n_phases, double eps_target, double delta,
                                  int max_alpha, double rel_tol, double* sigma) {
    if (!sigma) return DP_ERR_NULL;
    if (!(eps_target > 0.0) || !(rel_tol > 0.0 && rel_tol < 1.0)) return DP_ERR_VALUE;
    // the guarantee shrinks as sigma grows: bracket the target from sigma = 1 by doubling / halving, then bisect
    double e, hi = 1.0;
    for (;;) {
        const dp_status st = dp_rdp_epsilon(q, steps, n_phases, hi, delta, max_alpha, &e, nullptr);
        if (st != DP_OK) return st;
        if (e <= eps_target) break;
        hi *= 2.0;
        if (hi > 1048576.0) return DP_ERR_VALUE;  // the conversion term of the largest order alone is above the target
    }
    double lo = hi / 2.0;
    for (;;) {
        const dp_status st = dp_rdp_epsilon(q, steps, n_phases, lo, delta, max_alpha, &e, nullptr);
        if (st != DP_OK) return st;
        if (e > eps_target) break;
        hi = lo;
        lo = lo / 2.0;
        if (lo < 1.0 / 1024.0) {  // no noise to speak of is needed (no steps, or nothing is ever sampled)
            *sigma = hi;
            return DP_OK;
        }
    }
    while (hi - lo > rel_tol * hi) {
        const double mid = 0.5 * (lo + hi);
        const dp_status st = dp_rdp_epsilon(q, steps, n_phases, mid, delta, max_alpha, &e, nullptr);
        if (st != DP_OK) return st;
        if (e <= eps_target) hi = mid;
        else lo = mid;
    }
    *sigma = hi;
    return DP_OK;
}

dp_status dp_sqnorms_dense(dp_ctx* ctx, const void* A, const void* G, dp_dtype dtype, int B, int T, int d_in,
                           int d_out, int has_bias, dp_path path, float* sqnorms) {
    REQUIRE_CTX(ctx);
    TRY(check_dtype(ctx, dtype));
    if (path != DP_PATH_AUTO && path != DP_PATH_GRAM && path != DP_PATH_MATERIALISE)
        FAIL(ctx, DP_ERR_DTYPE, "unknown path %d", (int)path);
    TRY(check_bt(ctx, B, T));
    if (d_in < 0 || d_out < 0) FAIL(ctx, DP_ERR_SHAPE, "negative layer width");
    TRY(check_tensor(ctx, "A", A, dtype, d_in));
    TRY(check_tensor(ctx, "G", G, dtype, d_out));
    TRY(check_f32(ctx, "sqnorms", sqnorms));
    if (B == 0 || T == 0 || d_out == 0) return DP_OK;
    if (d_in == 0) {  // no weights; only the bias term is left
        if (has_bias) return dpk_colstat_sqnorms(ctx, nullptr, G, dtype, B, T, d_out, 0, 1, sqnorms);
        return DP_OK;
    }
    if (path == DP_PATH_AUTO) dp_choose_path(T, d_in, d_out, dtype, &path);
    if (path == DP_PATH_GRAM) return dpk_gram_sqnorms(ctx, A, G, dtype, B, T, d_in, d_out, has_bias, sqnorms);
    return dpk_materialise_sqnorms(ctx, A, G, dtype, B, T, d_in, d_out, has_bias, sqnorms);
}

dp_status dp_sqnorms_dense_batched(dp_ctx* ctx, int n_layers, const void* const* A, const void* const* G, dp_dtype dtype,
                                   int B, int T, int d_in, int d_out, int has_bias, dp_path path, float* sqnorms) {
    REQUIRE_CTX(ctx);
    TRY(check_dtype(ctx, dtype));
    if (path != DP_PATH_AUTO && path != DP_PATH_GRAM && path != DP_PATH_MATERIALISE)
        FAIL(ctx, DP_ERR_DTYPE, "unknown path %d", (int)path);
    TRY(check_bt(ctx, B, T));
    if (n_layers < 0 || d_in < 0 || d_out < 0) FAIL(ctx, DP_ERR_SHAPE, "negative layer count or width");
    if (n_layers == 0) return DP_OK;
    if (!A || !G) FAIL(ctx, DP_ERR_NULL, "a pointer table is NULL");
    for (int l = 0; l < n_layers; ++l) {
        TRY(check_tensor(ctx, "A[l]", A[l], dtype, d_in));
        TRY(check_tensor(ctx, "G[l]", G[l], dtype, d_out));
    }
    TRY(check_f32(ctx, "sqnorms", sqnorms));
    if (B == 0 || T == 0 || d_out == 0) return DP_OK;
    if (path == DP_PATH_AUTO && d_in > 0) dp_choose_path(T, d_in, d_out, dtype, &path);
    if (path == DP_PATH_GRAM && d_in > 0)
        return dpk_gram_sqnorms_batched(ctx, n_layers, A, G, dtype, B, T, d_in, d_out, has_bias, sqnorms);
    for (int l = 0; l < n_layers; ++l)
        TRY(dp_sqnorms_dense(ctx, A[l], G[l], dtype, B, T, d_in, d_out, has_bias, path, sqnorms));
    return DP_OK;
}

dp_status dp_sqnorms_dense_shared(dp_ctx* ctx, int n_groups, const void* const* A, int n_out, const void* const* G,
                                  dp_dtype dtype, int B, int T, int d_in, int d_out, int has_bias, float* sqnorms) {
    REQUIRE_CTX(ctx);
    TRY(check_dtype(ctx, dtype));
    TRY(check_bt(ctx, B, T));
    if (n_groups < 0 || n_out < 1 || d_in < 0 || d_out < 0) FAIL(ctx, DP_ERR_SHAPE, "negative count or width");
    if (n_groups == 0) return DP_OK;
    if (!A || !G) FAIL(ctx, DP_ERR_NULL, "a pointer table is NULL");
    for (int g = 0; g < n_groups; ++g) {
        TRY(check_tensor(ctx, "A[g]", A[g], dtype, d_in));
        for (int j = 0; j < n_out; ++j) TRY(check_tensor(ctx, "G[g][j]", G[(size_t)g * n_out + j], dtype, d_out));
    }
    TRY(check_f32(ctx, "sqnorms", sqnorms));
    if (B == 0 || T == 0 || d_out == 0) return DP_OK;
    dp_path path = DP_PATH_GRAM;
    if (d_in > 0) dp_choose_path(T, d_in, n_out * d_out, dtype, &path);  // one A A^T serves n_out output Grams
    if (d_in > 0 && path == DP_PATH_GRAM)
        return dpk_gram_sqnorms_shared(ctx, n_groups, A, n_out, G, dtype, B, T, d_in, d_out, has_bias, sqnorms);
    for (int g = 0; g < n_groups; ++g)
        for (int j = 0; j < n_out; ++j)
            TRY(dp_sqnorms_dense(ctx, A[g], G[(size_t)g * n_out + j], dtype, B, T, d_in, d_out, has_bias, DP_PATH_AUTO, sqnorms));
    return DP_OK;
}

dp_status dp_sqnorms_layernorm(dp_ctx* ctx, const void* Xhat, const void* G, dp_dtype dtype, int B, int T, int d,
                               float* sqnorms) {
    REQUIRE_CTX(ctx);
    TRY(check_dtype(ctx, dtype));
    TRY(check_bt(ctx, B, T));
    if (d < 0) FAIL(ctx, DP_ERR_SHAPE, "negative width");
    TRY(check_tensor(ctx, "Xhat", Xhat, dtype, d));
    TRY(check_tensor(ctx, "G", G, dtype, d));
    TRY(check_f32(ctx, "sqnorms", sqnorms));
    return dpk_colstat_sqnorms(ctx, Xhat, G, dtype, B, T, d, 1, 1, sqnorms);
}

dp_status dp_sqnorms_embedding(dp_ctx* ctx, const int32_t* ids, const void* G, dp_dtype dtype, int B, int T, int d,
                               int V, int distinct_per_example, float* sqnorms) {
    REQUIRE_CTX(ctx);
    TRY(check_dtype(ctx, dtype));
    TRY(check_bt(ctx, B, T));
    if (d < 0 || V <= 0) FAIL(ctx, DP_ERR_SHAPE, "width must be >= 0 and V > 0");
    TRY(check_f32(ctx, "ids", ids));
    TRY(check_tensor(ctx, "G", G, dtype, d));
    TRY(check_f32(ctx, "sqnorms", sqnorms));
    return dpk_embedding_sqnorms(ctx, ids, G, dtype, B, T, d, V, distinct_per_example, sqnorms);
}

dp_status dp_clip_factors(dp_ctx* ctx, const float* sqnorms, int B, float C, float* c) {
    REQUIRE_CTX(ctx);
    if (B < 0) FAIL(ctx, DP_ERR_SHAPE, "negative B");
    TRY(check_f32(ctx, "sqnorms", sqnorms));
    TRY(check_f32(ctx, "c", c));
    if (!(C > 0.f) || !isfinite(C)) FAIL(ctx, DP_ERR_VALUE, "clip norm C must be positive and finite");
    if (B == 0) return DP_OK;
    return dpk_clip_factors(ctx, sqnorms, B, C, c);
}

dp_status dp_clip_accumulate_dense(dp_ctx* ctx, const void* A, const void* G, dp_dtype dtype, int B, int T, int d_in,
                                   int d_out, float C, const float* sqnorms, float* sum_W, float* sum_b) {
    REQUIRE_CTX(ctx);
    TRY(check_dtype(ctx, dtype));
    TRY(check_bt(ctx, B, T));
    if (d_in < 0 || d_out < 0) FAIL(ctx, DP_ERR_SHAPE, "negative layer width");
    TRY(check_tensor(ctx, "A", A, dtype, d_in));
    TRY(check_tensor(ctx, "G", G, dtype, d_out));
    TRY(check_f32(ctx, "sqnorms", sqnorms));
    TRY(check_f32(ctx, "sum_W", sum_W));
    if (sum_b) TRY(check_f32(ctx, "sum_b", sum_b));
    if (dtype == DP_BF16 && ((uintptr_t)sum_W & 15)) FAIL(ctx, DP_ERR_ALIGN, "sum_W is not 16-byte aligned");
    TRY(check_clip(ctx, C, B));
    if (B == 0 || T == 0 || d_out == 0) return DP_OK;
    return dpk_weighted_gemm(ctx, A, G, dtype, B, T, d_in, d_out, sqnorms, C, sum_W, sum_b);
}

dp_status dp_clip_accumulate_dense_batched(dp_ctx* ctx, int n_layers, const void* const* A, const void* const* G,
                                           dp_dtype dtype, int B, int T, int d_in, int d_out, float C,
                                           const float* sqnorms, float* const* sum_W, float* const* sum_b) {
    REQUIRE_CTX(ctx);
    TRY(check_dtype(ctx, dtype));
    TRY(check_bt(ctx, B, T));
    if (n_layers < 0 || d_in < 0 || d_out < 0) FAIL(ctx, DP_ERR_SHAPE, "negative layer count or width");
    if (n_layers == 0) return DP_OK;
    if (!A || !G || !sum_W) FAIL(ctx, DP_ERR_NULL, "a pointer table is NULL");
    for (int l = 0; l < n_layers; ++l) {
        TRY(check_tensor(ctx, "A[l]", A[l], dtype, d_in));
        TRY(check_tensor(ctx, "G[l]", G[l], dtype, d_out));
        TRY(check_f32(ctx, "sum_W[l]", sum_W[l]));
        if (dtype == DP_BF16 && ((uintptr_t)sum_W[l] & 15)) FAIL(ctx, DP_ERR_ALIGN, "sum_W[%d] is not 16-byte aligned", l);
        if (sum_b && sum_b[l]) TRY(check_f32(ctx, "sum_b[l]", sum_b[l]));
    }
    TRY(check_f32(ctx, "sqnorms", sqnorms));
    TRY(check_clip(ctx, C, B));
    if (B == 0 || T == 0 || d_out == 0) return DP_OK;
    return dpk_weighted_gemm_batched(ctx, n_layers, A, G, dtype, B, T, d_in, d_out, sqnorms, C, sum_W, sum_b);
}

dp_status dp_clip_accumulate_layernorm(dp_ctx* ctx, const void* Xhat, const void* G, dp_dtype dtype, int B, int T,
                                       int d, float C, const float* sqnorms, float* sum_gamma, float* sum_beta) {
    REQUIRE_CTX(ctx);
    TRY(check_dtype(ctx, dtype));
    TRY(check_bt(ctx, B, T));
    if (d < 0) FAIL(ctx, DP_ERR_SHAPE, "negative width");
    TRY(check_tensor(ctx, "Xhat", Xhat, dtype, d));
    TRY(check_tensor(ctx, "G", G, dtype, d));
    TRY(check_f32(ctx, "sqnorms", sqnorms));
    TRY(check_f32(ctx, "sum_gamma", sum_gamma));
    TRY(check_f32(ctx, "sum_beta", sum_beta));
    TRY(check_clip(ctx, C, B));
    if (B == 0 || T == 0 || d == 0) return DP_OK;
    TRY(dpk_clip_factors(ctx, sqnorms, B, C, ctx->cbuf));
    return dpk_colstat_sums(ctx, Xhat, G, dtype, B, T, d, ctx->cbuf, sum_gamma, sum_beta);
}

dp_status dp_sqnorms_layernorm_batched(dp_ctx* ctx, int n_layers, const void* const* Xhat, const void* const* G,
                                       dp_dtype dtype, int B, int T, int d, float* sqnorms) {
    REQUIRE_CTX(ctx);
    TRY(check_dtype(ctx, dtype));
    TRY(check_bt(ctx, B, T));
    if (n_layers < 0 || d < 0) FAIL(ctx, DP_ERR_SHAPE, "negative layer count or width");
    if (n_layers == 0) return DP_OK;
    if (!Xhat || !G) FAIL(ctx, DP_ERR_NULL, "a pointer table is NULL");
    for (int l = 0; l < n_layers; ++l) {
        TRY(check_tensor(ctx, "Xhat[l]", Xhat[l], dtype, d));
        TRY(check_tensor(ctx, "G[l]", G[l], dtype, d));
    }
    TRY(check_f32(ctx, "sqnorms", sqnorms));
    return dpk_colstat_sqnorms_batched(ctx, n_layers, Xhat, G, dtype, B, T, d, 1, 1, sqnorms, nullptr);
}

dp_status dp_sqnorms_layernorm_keep(dp_ctx* ctx, int n_layers, const void* const* Xhat, const void* const* G, dp_dtype dtype,
                                    int B, int T, int d, float* sqnorms, float* const* grads) {
    REQUIRE_CTX(ctx);
    TRY(check_dtype(ctx, dtype));
    TRY(check_bt(ctx, B, T));
    if (n_layers < 0 || d < 0) FAIL(ctx, DP_ERR_SHAPE, "negative layer count or width");
    if (d % 4) FAIL(ctx, DP_ERR_SHAPE, "width %d is not a multiple of 4", d);
    if (n_layers == 0) return DP_OK;
    if (!Xhat || !G || !grads) FAIL(ctx, DP_ERR_NULL, "a pointer table is NULL");
    for (int l = 0; l < n_layers; ++l) {
        TRY(check_tensor(ctx, "Xhat[l]", Xhat[l], dtype, d));
        TRY(check_tensor(ctx, "G[l]", G[l], dtype, d));
        TRY(check_f32(ctx, "grads[l]", grads[l]));
        if ((uintptr_t)grads[l] & 15) FAIL(ctx, DP_ERR_ALIGN, "grads[%d] is not 16-byte aligned", l);
    }
    TRY(check_f32(ctx, "sqnorms", sqnorms));
    if (B == 0 || d == 0) return DP_OK;
    if (T == 0) {  // no tokens: every example's gradient is zero
        for (int l = 0; l < n_layers; ++l) TRY(dpk_zero_f32(ctx, grads[l], (uint64_t)B * 2 * d));
        return DP_OK;
    }
    return dpk_colstat_sqnorms_batched(ctx, n_layers, Xhat, G, dtype, B, T, d, 1, 1, sqnorms, grads);
}

dp_status dp_clip_accumulate_layernorm_kept(dp_ctx* ctx, int n_layers, float* const* grads, int B, int d, float C,
                                            const float* sqnorms, float* const* sum_gamma, float* const* sum_beta) {
    REQUIRE_CTX(ctx);
    if (B < 0 || n_layers < 0 || d < 0) FAIL(ctx, DP_ERR_SHAPE, "negative count or width");
    if (d % 4) FAIL(ctx, DP_ERR_SHAPE, "width %d is not a multiple of 4", d);
    if (n_layers == 0) return DP_OK;
    if (!grads || !sum_gamma || !sum_beta) FAIL(ctx, DP_ERR_NULL, "a pointer table is NULL");
    for (int l = 0; l < n_layers; ++l) {
        TRY(check_f32(ctx, "grads[l]", grads[l]));
        TRY(check_f32(ctx, "sum_gamma[l]", sum_gamma[l]));
        TRY(check_f32(ctx, "sum_beta[l]", sum_beta[l]));
        if (((uintptr_t)grads[l] | (uintptr_t)sum_gamma[l] | (uintptr_t)sum_beta[l]) & 15)
            FAIL(ctx, DP_ERR_ALIGN, "grads, sum_gamma and sum_beta must be 16-byte aligned (layer %d)", l);
    }
    TRY(check_f32(ctx, "sqnorms", sqnorms));
    TRY(check_clip(ctx, C, B));
    if (B == 0 || d == 0) return DP_OK;
    TRY(dpk_clip_factors(ctx, sqnorms, B, C, ctx->cbuf));
    return dpk_kept_sums_batched(ctx, n_layers, grads, B, d, ctx->cbuf, sum_gamma, sum_beta);
}

dp_status dp_clip_accumulate_layernorm_batched(dp_ctx* ctx, int n_layers, const void* const* Xhat, const void* const* G,
                                               dp_dtype dtype, int B, int T, int d, float C, const float* sqnorms,
                                               float* const* sum_gamma, float* const* sum_beta) {
    REQUIRE_CTX(ctx);
    TRY(check_dtype(ctx, dtype));
    TRY(check_bt(ctx, B, T));
    if (n_layers < 0 || d < 0) FAIL(ctx, DP_ERR_SHAPE, "negative layer count or width");
    if (n_layers == 0) return DP_OK;
    if (!Xhat || !G || !sum_gamma || !sum_beta) FAIL(ctx, DP_ERR_NULL, "a pointer table is NULL");
    for (int l = 0; l < n_layers; ++l) {
        TRY(check_tensor(ctx, "Xhat[l]", Xhat[l], dtype, d));
        TRY(check_tensor(ctx, "G[l]", G[l], dtype, d));
        TRY(check_f32(ctx, "sum_gamma[l]", sum_gamma[l]));
        TRY(check_f32(ctx, "sum_beta[l]", sum_beta[l]));
    }
    TRY(check_f32(ctx, "sqnorms", sqnorms));
    TRY(check_clip(ctx, C, B));
    if (B == 0 || T == 0 || d == 0) return DP_OK;
    TRY(dpk_clip_factors(ctx, sqnorms, B, C, ctx->cbuf));
    return dpk_colstat_sums_batched(ctx, n_layers, Xhat, G, dtype, B, T, d, ctx->cbuf, sum_gamma, sum_beta);
}

dp_status dp_clip_accumulate_embedding(dp_ctx* ctx, const int32_t* ids, const void* G, dp_dtype dtype, int B, int T,
                                       int d, int V, float C, const float* sqnorms, float* sum_E) {
    REQUIRE_CTX(ctx);
    TRY(check_dtype(ctx, dtype));
    TRY(check_bt(ctx, B, T));
    if (d < 0 || V <= 0) FAIL(ctx, DP_ERR_SHAPE, "width must be >= 0 and V > 0");
    TRY(check_f32(ctx, "ids", ids));
    TRY(check_tensor(ctx, "G", G, dtype, d));
    TRY(check_f32(ctx, "sqnorms", sqnorms));
    TRY(check_f32(ctx, "sum_E", sum_E));
    TRY(check_clip(ctx, C, B));
    if (B == 0 || T == 0 || d == 0) return DP_OK;
    TRY(dpk_clip_factors(ctx, sqnorms, B, C, ctx->cbuf));
    return dpk_embedding_sums(ctx, ids, G, dtype, B, T, d, V, ctx->cbuf, sum_E);
}

dp_status dp_clip_accumulate_positions(dp_ctx* ctx, const void* G, dp_dtype dtype, int B, int T, int d, float C,
                                       const float* sqnorms, float* sum_E) {
    REQUIRE_CTX(ctx);
    TRY(check_dtype(ctx, dtype));
    TRY(check_bt(ctx, B, T));
    if (d < 0) FAIL(ctx, DP_ERR_SHAPE, "width must be >= 0");
    TRY(check_tensor(ctx, "G", G, dtype, d));
    TRY(check_f32(ctx, "sqnorms", sqnorms));
    TRY(check_f32(ctx, "sum_E", sum_E));
    TRY(check_clip(ctx, C, B));
    if (B == 0 || T == 0 || d == 0) return DP_OK;
    if ((long)T * d > 0x7FFFFFFFl) FAIL(ctx, DP_ERR_SHAPE, "T * d too large");
    TRY(dpk_clip_factors(ctx, sqnorms, B, C, ctx->cbuf));
    // token t of every example adds to row t: the first T rows of the table, read as one vector of T*d entries,
    // receive sum_i c_i * (example i's gradient read as one row of T*d entries): a weighted column sum over B rows
    return dpk_colstat_sums(ctx, nullptr, G, dtype, B, 1, T * d, ctx->cbuf, nullptr, sum_E);
}

static dp_status check_tied(dp_ctx* ctx, const int32_t* ids, const void* dY, const void* H, const void* dL,
                            dp_dtype dtype, int B, int T, int M, int d, int V, const float* sqnorms) {
    TRY(check_dtype(ctx, dtype));
    TRY(check_bt(ctx, B, T));
    TRY(check_bt(ctx, B, M));
    if (d < 0 || V <= 0) FAIL(ctx, DP_ERR_SHAPE, "width must be >= 0 and V > 0");
    if ((long)M * V > (long)INT_MAX) FAIL(ctx, DP_ERR_SHAPE, "M * V = %ld exceeds 2^31", (long)M * V);
    TRY(check_f32(ctx, "ids", ids));
    TRY(check_tensor(ctx, "dY", dY, dtype, d));
    if (M > 0) {
        TRY(check_tensor(ctx, "H", H, dtype, d));
        TRY(check_tensor(ctx, "dL", dL, dtype, V));
    }
    TRY(check_f32(ctx, "sqnorms", sqnorms));
    return DP_OK;
}

dp_status dp_sqnorms_tied_embedding(dp_ctx* ctx, const int32_t* ids, const void* dY, const void* H, const void* dL,
                                    dp_dtype dtype, int B, int T, int M, int d, int V, float* sqnorms) {
    REQUIRE_CTX(ctx);
    TRY(check_tied(ctx, ids, dY, H, dL, dtype, B, T, M, d, V, sqnorms));
    if (B == 0 || d == 0) return DP_OK;
    if (T > 0) TRY(dpk_embedding_sqnorms(ctx, ids, dY, dtype, B, T, d, V, 0, sqnorms));
    if (M == 0) return DP_OK;
    // the output projection as a dense layer with weight E: "input" dL_i [M, V], "output gradient" H_i [M, d];
    // M is far below both widths, so the Gram form <dL dL^T, H H^T> is the cheap one
    TRY(dpk_gram_sqnorms(ctx, dL, H, dtype, B, M, V, d, 0, sqnorms));
    return dpk_tied_cross_sqnorms(ctx, ids, dY, H, dL, dtype, B, T, M, d, V, sqnorms);
}

dp_status dp_clip_accumulate_tied_embedding(dp_ctx* ctx, const int32_t* ids, const void* dY, const void* H,
                                            const void* dL, dp_dtype dtype, int B, int T, int M, int d, int V, float C,
                                            const float* sqnorms, float* sum_E) {
    REQUIRE_CTX(ctx);
    TRY(check_tied(ctx, ids, dY, H, dL, dtype, B, T, M, d, V, sqnorms));
    TRY(check_f32(ctx, "sum_E", sum_E));
    if (dtype == DP_BF16 && ((uintptr_t)sum_E & 15)) FAIL(ctx, DP_ERR_ALIGN, "sum_E is not 16-byte aligned");
    TRY(check_clip(ctx, C, B));
    if (B == 0 || d == 0) return DP_OK;
    if (T > 0) {
        TRY(dpk_clip_factors(ctx, sqnorms, B, C, ctx->cbuf));
        TRY(dpk_embedding_sums(ctx, ids, dY, dtype, B, T, d, V, ctx->cbuf, sum_E));
    }
    if (M == 0) return DP_OK;
    return dpk_tied_projection_sums(ctx, H, dL, dtype, B, M, d, V, sqnorms, C, sum_E);
}

// Argument checks of the update; *why is set to a static text on failure.
static dp_status check_update_args(const float* params, const float* m, const float* v, const float* sum, uint64_t n,
                                   uint64_t elem_offset, float sigma, float C, uint64_t step, uint64_t batch_size, float lr,
                                   float beta1, float beta2, float eps, float weight_decay, const char** why) {
#define UPD_FAIL(code, text) \
    do {                     \
        *why = text;         \
        return code;         \
    } while (0)
    if (!params || !m || !v || !sum) UPD_FAIL(DP_ERR_NULL, "params, m, v or sum is NULL");
    if (((uintptr_t)params | (uintptr_t)m | (uintptr_t)v | (uintptr_t)sum) & 3) UPD_FAIL(DP_ERR_ALIGN, "params, m, v and sum must be 4-byte aligned");
    if (!(sigma >= 0.f) || !isfinite(sigma)) UPD_FAIL(DP_ERR_VALUE, "sigma must be >= 0 and finite");
    if (!(C > 0.f) || !isfinite(C)) UPD_FAIL(DP_ERR_VALUE, "clip norm C must be positive and finite");
    if (batch_size == 0) UPD_FAIL(DP_ERR_VALUE, "batch_size must be positive");
    if (step == 0) UPD_FAIL(DP_ERR_VALUE, "step counts from 1");
    if (!(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f)) UPD_FAIL(DP_ERR_VALUE, "beta outside [0, 1)");
    if (!(eps >= 0.f) || !isfinite(eps)) UPD_FAIL(DP_ERR_VALUE, "eps must be >= 0 and finite");
    if (!isfinite(lr) || !isfinite(weight_decay)) UPD_FAIL(DP_ERR_VALUE, "lr and weight_decay must be finite");
    if (elem_offset + n < elem_offset) UPD_FAIL(DP_ERR_SHAPE, "elem_offset + n overflows");
#undef UPD_FAIL
    return DP_OK;
}

static dp_status noise_adamw_checked(dp_ctx* ctx, float* params, float* m, float* v, float* sum, uint64_t n,
                                     uint64_t elem_offset, float sigma, float C, uint64_t seed, uint64_t step,
                                     uint64_t batch_size, float lr, float beta1, float beta2, float eps,
                                     float weight_decay, int zero_sum, float* sq_out) {
    const char* why = "";
    const dp_status st = check_update_args(params, m, v, sum, n, elem_offset, sigma, C, step, batch_size, lr, beta1, beta2,
                                           eps, weight_decay, &why);
    if (st != DP_OK) FAIL(ctx, st, "%s", why);
    return dpk_noise_adamw(ctx, params, m, v, sum, n, elem_offset, sigma, C, seed, step, batch_size, lr, beta1, beta2,
                           eps, weight_decay, zero_sum, sq_out);
}

dp_status dp_noise_adamw(dp_ctx* ctx, float* params, float* m, float* v, float* sum, uint64_t n,
                         uint64_t elem_offset, float sigma, float C, uint64_t seed, uint64_t step,
                         uint64_t batch_size, float lr, float beta1, float beta2, float eps, float weight_decay,
                         int zero_sum) {
    REQUIRE_CTX(ctx);
    return noise_adamw_checked(ctx, params, m, v, sum, n, elem_offset, sigma, C, seed, step, batch_size, lr, beta1,
                               beta2, eps, weight_decay, zero_sum, nullptr);
}

dp_status dp_noise_adamw_snr(dp_ctx* ctx, float* params, float* m, float* v, float* sum, uint64_t n,
                             uint64_t elem_offset, float sigma, float C, uint64_t seed, uint64_t step,
                             uint64_t batch_size, float lr, float beta1, float beta2, float eps, float weight_decay,
                             int zero_sum, float* snr_sq) {
    REQUIRE_CTX(ctx);
    if (!snr_sq) FAIL(ctx, DP_ERR_NULL, "snr_sq is NULL");
    if ((uintptr_t)snr_sq & 3) FAIL(ctx, DP_ERR_ALIGN, "snr_sq must be 4-byte aligned");
    return noise_adamw_checked(ctx, params, m, v, sum, n, elem_offset, sigma, C, seed, step, batch_size, lr, beta1,
                               beta2, eps, weight_decay, zero_sum, snr_sq);
}

dp_status dp_noise_adamw_snr_static(void* hip_stream, float* params, float* m, float* v, float* sum, uint64_t n,
                                    uint64_t elem_offset, float sigma, float C, uint64_t seed, uint64_t step,
                                    uint64_t batch_size, float lr, float beta1, float beta2, float eps, float weight_decay,
                                    int zero_sum, float* snr_sq) {
    if (!snr_sq) return DP_ERR_NULL;
    if ((uintptr_t)snr_sq & 3) return DP_ERR_ALIGN;
    const char* why = "";
    const dp_status st = check_update_args(params, m, v, sum, n, elem_offset, sigma, C, step, batch_size, lr, beta1, beta2,
                                           eps, weight_decay, &why);
    if (st != DP_OK) return st;
    return dpk_noise_adamw_snr_static((hipStream_t)hip_stream, params, m, v, sum, n, elem_offset, sigma, C, seed, step,
                                      batch_size, lr, beta1, beta2, eps, weight_decay, zero_sum, snr_sq);
}

dp_status dp_zero_f32(dp_ctx* ctx, float* p, uint64_t n) {
    REQUIRE_CTX(ctx);
    TRY(check_f32(ctx, "p", p));
    return dpk_zero_f32(ctx, p, n);
}

dp_status dp_philox_u32(dp_ctx* ctx, uint32_t* out, uint64_t n, uint64_t elem_offset, uint64_t seed, uint64_t step) {
    REQUIRE_CTX(ctx);
    TRY(check_f32(ctx, "out", out));
    if (elem_offset + n < elem_offset) FAIL(ctx, DP_ERR_SHAPE, "elem_offset + n overflows");
    return dpk_philox_u32(ctx, out, n, elem_offset, seed, step);
}

dp_status dp_normal_f32(dp_ctx* ctx, float* out, uint64_t n, uint64_t elem_offset, uint64_t seed, uint64_t step) {
    REQUIRE_CTX(ctx);
    TRY(check_f32(ctx, "out", out));
    if (elem_offset + n < elem_offset) FAIL(ctx, DP_ERR_SHAPE, "elem_offset + n overflows");
    return dpk_normal_f32(ctx, out, n, elem_offset, seed, step);
}

}  // extern "C"
