// Internal declarations shared by the HIP sources of libdpclip (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "dpclip.h"

struct dp_prof_rec {
    hipEvent_t start, stop;
    int kind;
    double work;
};
constexpr int DP_PROF_CAP = 65536;

struct dp_ctx {
    hipStream_t stream;
    int device;
    char* ws;         // device workspace
    size_t ws_bytes;
    size_t ws_base;   // bytes at the start of the workspace held by an enclosing step of the current call
    int* err_word;    // device: bit 0 = token id out of range, bit 1 = a squared norm that is not a finite number
    float* cbuf;      // device: clip factors of the current micro-batch
    int cbuf_cap;     // capacity of cbuf in floats
    int prof_on;
    dp_prof_rec* prof;  // DP_PROF_CAP records; events are created on first use and reused
    int prof_n;         // records in use
    int prof_made;      // records whose events exist
    char msg[256];
};

// Brackets one kernel launch with events when profiling is on (no-op otherwise).
struct dp_prof_scope {
    dp_ctx* ctx;
    dp_prof_rec* rec;
    dp_prof_scope(dp_ctx* c, int kind, double work) : ctx(c), rec(nullptr) {
        if (!c->prof_on || c->prof_n >= DP_PROF_CAP) return;
        dp_prof_rec* r = &c->prof[c->prof_n];
        if (c->prof_n >= c->prof_made) {
            if (hipEventCreate(&r->start) != hipSuccess) return;
            if (hipEventCreate(&r->stop) != hipSuccess) { (void)hipEventDestroy(r->start); return; }
            c->prof_made = c->prof_n + 1;
        }
        r->kind = kind;
        r->work = work;
        if (hipEventRecord(r->start, c->stream) != hipSuccess) return;
        rec = r;
        c->prof_n++;
    }
    ~dp_prof_scope() {
        if (rec) (void)hipEventRecord(rec->stop, ctx->stream);
    }
};

#define DP_SET_ERR(ctx, ...) snprintf((ctx)->msg, sizeof((ctx)->msg), __VA_ARGS__)

#define DP_HIP_CHECK(ctx, expr)                                                      \
    do {                                                                             \
        hipError_t e__ = (expr);                                                     \
        if (e__ != hipSuccess) {                                                     \
            DP_SET_ERR(ctx, "%s failed: %s", #expr, hipGetErrorString(e__));         \
            return DP_ERR_HIP;                                                       \
        }                                                                            \
    } while (0)

#define DP_LAUNCH_CHECK(ctx, what)                                                   \
    do {                                                                             \
        hipError_t e__ = hipGetLastError();                                          \
        if (e__ != hipSuccess) {                                                     \
            DP_SET_ERR(ctx, "launch of %s failed: %s", what, hipGetErrorString(e__)); \
            return DP_ERR_HIP;                                                       \
        }                                                                            \
    } while (0)

static inline size_t dp_align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Simple bump allocator over the context workspace (valid for the duration of one API call:
// all kernels of a call run on one stream before those of the next call).
struct dp_ws_alloc {
    dp_ctx* ctx;
    size_t off;
    explicit dp_ws_alloc(dp_ctx* c) : ctx(c), off(c->ws_base) {}
    template <typename T>
    T* get(size_t count) {
        size_t o = dp_align_up(off, 256);
        size_t end = o + count * sizeof(T);
        if (end > ctx->ws_bytes) return nullptr;
        off = end;
        return reinterpret_cast<T*>(ctx->ws + o);
    }
    size_t remaining() const {
        size_t o = dp_align_up(off, 256);
        return o >= ctx->ws_bytes ? 0 : ctx->ws_bytes - o;
    }
};

// Keeps what `a` has handed out so far while launchers called inside the scope take workspace of their own.
struct dp_ws_hold {
    dp_ctx* ctx;
    size_t saved;
    explicit dp_ws_hold(const dp_ws_alloc& a) : ctx(a.ctx), saved(a.ctx->ws_base) { ctx->ws_base = dp_align_up(a.off, 256); }
    ~dp_ws_hold() { ctx->ws_base = saved; }
};

// ------------------------------------------------------------------------------------------------
// device helpers
// ------------------------------------------------------------------------------------------------
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float dp_bf16_bits_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }
__device__ __forceinline__ float dp_bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float dp_bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// fp32 -> bf16 bits, round to nearest even (inputs here are finite products c*g).
__device__ __forceinline__ uint32_t dp_f32_to_bf16_bits(float x) {
    uint32_t u = __float_as_uint(x);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ uint32_t dp_pack_bf16x2(float lo, float hi) {
    return dp_f32_to_bf16_bits(lo) | (dp_f32_to_bf16_bits(hi) << 16);
}

__device__ __forceinline__ float dp_wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// Sum over a workgroup of NT threads (NT multiple of 64, <= 1024); result valid in thread 0.
// `red` is LDS scratch of at least NT/64 floats.  Fixed order => deterministic.
template <int NT>
__device__ __forceinline__ float dp_block_sum(float v, float* red) {
    v = dp_wave_sum(v);
    const int w = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    float t = 0.f;
    if (threadIdx.x == 0) {
#pragma unroll
        for (int i = 0; i < NT / 64; ++i) t += red[i];
    }
    return t;
}

constexpr int DP_ERRBIT_INDEX = 1, DP_ERRBIT_NORM = 2;

__device__ __forceinline__ float dp_clip_factor(float sqnorm, float C) {
    // c = min(1, C / ||g||); a zero gradient keeps factor 1.  A squared norm that is NaN or overflowed fp32 has no
    // clip factor: NaN, on every path alike, so that the sums it enters are NaN too (and dp_sync reports it).
    if (!(sqnorm < __builtin_inff())) return __builtin_nanf("");
    return sqnorm > 0.f ? fminf(1.f, C / sqrtf(sqnorm)) : 1.f;
}

// ------------------------------------------------------------------------------------------------
// launchers implemented in the .hip files (host side; all enqueue on ctx->stream)
// ------------------------------------------------------------------------------------------------
dp_status dpk_zero_f32(dp_ctx*, float* p, uint64_t n);
dp_status dpk_finish_partials(dp_ctx*, const float* partial, int B, int J, float* sqnorms);
dp_status dpk_clip_factors(dp_ctx*, const float* sqnorms, int B, float C, float* c);
dp_status dpk_reduce_partials(dp_ctx*, const float* part, int R, size_t stride, size_t n, float* out);
dp_status dpk_materialise_f32(dp_ctx*, const float* A, const float* G, int B, int T, int d_in, int d_out,
                              float* sqnorms);

dp_status dpk_philox_u32(dp_ctx*, uint32_t* out, uint64_t n, uint64_t off, uint64_t seed, uint64_t step);
dp_status dpk_normal_f32(dp_ctx*, float* out, uint64_t n, uint64_t off, uint64_t seed, uint64_t step);
dp_status dpk_noise_adamw(dp_ctx*, float* params, float* m, float* v, float* sum, uint64_t n, uint64_t off,
                          float sigma, float C, uint64_t seed, uint64_t step, uint64_t batch, float lr, float b1,
                          float b2, float eps, float wd, int zero_sum, float* snr_sq /* device [2], += ; or NULL */);

dp_status dpk_static_scratch(float** out);
dp_status dpk_noise_adamw_snr_static(hipStream_t stream, float* params, float* m, float* v, float* sum, uint64_t n,
                                     uint64_t off, float sigma, float C, uint64_t seed, uint64_t step, uint64_t batch,
                                     float lr, float b1, float b2, float eps, float wd, int zero_sum, float* sq_out);

dp_status dpk_gram_unit_plan(int T, uint32_t* units, int capacity, int* n_units);
dp_status dpk_gram_sqnorms_batched(dp_ctx*, int n_layers, const void* const* A, const void* const* G, dp_dtype, int B, int T,
                                   int d_in, int d_out, int has_bias, float* sqnorms);
dp_status dpk_gram_sqnorms_shared(dp_ctx*, int n_groups, const void* const* A, int n_out, const void* const* G, dp_dtype, int B,
                                  int T, int d_in, int d_out, int has_bias, float* sqnorms);
dp_status dpk_gram_sqnorms(dp_ctx*, const void* A, const void* G, dp_dtype, int B, int T, int d_in, int d_out,
                           int has_bias, float* sqnorms);
dp_status dpk_materialise_sqnorms(dp_ctx*, const void* A, const void* G, dp_dtype, int B, int T, int d_in, int d_out,
                                  int has_bias, float* sqnorms);
// sum_W += sum_i c_i A_i^T G_i and, if sum_b, sum_b += sum_i c_i sum_t G_i[t,:], with c_i from (sqnorms, C)
dp_status dpk_weighted_gemm(dp_ctx*, const void* A, const void* G, dp_dtype, int B, int T, int d_in, int d_out,
                            const float* sqnorms, float C, float* sum_W, float* sum_b);

dp_status dpk_mfma_ceiling(dp_ctx*, int iters, int launches, double* tflops);
dp_status dpk_weighted_gemm_batched(dp_ctx*, int n, const void* const* A, const void* const* G, dp_dtype, int B, int T,
                                    int d_in, int d_out, const float* sqnorms, float C, float* const* sum_W,
                                    float* const* sum_b);

// column statistics shared by LayerNorm and dense-bias terms:
//   sqnorms:  n[i] += [use_x] sum_j (sum_t g x)^2 + [use_1] sum_j (sum_t g)^2
//   sums:     out_x[j] += sum_i c_i sum_t g x ; out_1[j] += sum_i c_i sum_t g   (either may be NULL)
dp_status dpk_colstat_sqnorms(dp_ctx*, const void* X, const void* G, dp_dtype, int B, int T, int d, int use_x,
                              int use_1, float* sqnorms);
dp_status dpk_colstat_sums(dp_ctx*, const void* X, const void* G, dp_dtype, int B, int T, int d, const float* c,
                           float* out_x, float* out_1);

dp_status dpk_colstat_sqnorms_batched(dp_ctx*, int n, const void* const* X, const void* const* G, dp_dtype, int B, int T, int d,
                                      int use_x, int use_1, float* sqnorms, float* const* keep /* or NULL */);
dp_status dpk_kept_sums_batched(dp_ctx*, int n, float* const* keep, int B, int d, const float* c, float* const* sum_x,
                                float* const* sum_1);
dp_status dpk_colstat_sums_batched(dp_ctx*, int n, const void* const* X, const void* const* G, dp_dtype, int B, int T, int d,
                                   const float* c, float* const* out_x, float* const* out_1);

dp_status dpk_embedding_sqnorms(dp_ctx*, const int32_t* ids, const void* G, dp_dtype, int B, int T, int d, int V,
                                int distinct, float* sqnorms);
dp_status dpk_embedding_sums(dp_ctx*, const int32_t* ids, const void* G, dp_dtype, int B, int T, int d, int V,
                             const float* c, float* sum_E);
// sum_E += sum_i c_i dL_i^T H_i   (the output-projection part of a tied table's clip-weighted sum)
dp_status dpk_tied_projection_sums(dp_ctx*, const void* H, const void* dL, dp_dtype, int B, int M, int d, int V,
                                   const float* sqnorms, float C, float* sum_E);
dp_status dpk_tied_cross_sqnorms(dp_ctx*, const int32_t* ids, const void* dY, const void* H, const void* dL, dp_dtype,
                                 int B, int T, int M, int d, int V, float* sqnorms);
