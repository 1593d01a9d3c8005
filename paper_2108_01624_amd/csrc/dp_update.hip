// Noise + Adam-with-decoupled-weight-decay streaming kernel (Algorithm 1, g_t line to theta_t line),
// the counter-based Philox4x32-10 generator it draws from, and small utility kernels.
//
// Roofline: HBM.  Per parameter the kernel reads theta, m, v, sum (16 B) and writes theta, m, v (12 B),
// plus 4 B when it also clears the sum: 28 (32) algorithmic bytes.  One thread owns one Philox block,
// i.e. four consecutive elements, so every access is a 16-byte vector and a wave covers 1 KiB per array.
#include <mutex>

#include "dp_common.h"

// Scratch of dp_noise_adamw_snr_static (the entry point that allocates nothing): one pair of partial squared norms per
// workgroup of the update, 2 floats per 1024 elements, for slices of up to DP_STATIC_MAX_ELEMS elements.  Every GPU
// that loads the library holds its own copy (about 8 MiB) until the process ends.  In host code this name is only a
// handle for hipGetSymbolAddress: kernels get the device address that call returns.
constexpr uint64_t DP_STATIC_MAX_ELEMS = 1ull << 30;
constexpr uint64_t DP_STATIC_MAX_PAIRS = DP_STATIC_MAX_ELEMS / 1024 + 2;
static __device__ __align__(256) float dp_static_scratch[2 * DP_STATIC_MAX_PAIRS];

namespace {

constexpr uint32_t PHILOX_M0 = 0xD2511F53u;
constexpr uint32_t PHILOX_M1 = 0xCD9E8D57u;
constexpr uint32_t PHILOX_W0 = 0x9E3779B9u;
constexpr uint32_t PHILOX_W1 = 0xBB67AE85u;

struct u32x4 {
    uint32_t x, y, z, w;
};

// Philox-4x32 with ten rounds (Salmon, Moraes, Dror, Shaw, SC'11): each round multiplies words 0 and 2 by
// fixed odd constants, keeps the low halves as words 3 and 1 and xors the high halves with words 3 / 1 and
// the round key; the key advances by Weyl constants between rounds.
__device__ __forceinline__ u32x4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                               uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(PHILOX_M0, c0), lo0 = PHILOX_M0 * c0;
        const uint32_t hi1 = __umulhi(PHILOX_M1, c2), lo1 = PHILOX_M1 * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0;
        const uint32_t n2 = hi0 ^ c3 ^ k1;
        c0 = n0;
        c1 = lo1;
        c2 = n2;
        c3 = lo0;
        k0 += PHILOX_W0;
        k1 += PHILOX_W1;
    }
    return {c0, c1, c2, c3};
}

__device__ __forceinline__ u32x4 philox_block(uint64_t block, uint64_t seed, uint64_t step) {
    return philox4x32_10((uint32_t)block, (uint32_t)(block >> 32), (uint32_t)step, (uint32_t)(step >> 32),
                         (uint32_t)seed, (uint32_t)(seed >> 32));
}

// 23-bit uniform in (0,1): ((r >> 9) + 1/2) * 2^-23, exact in fp32.
__device__ __forceinline__ float u01(uint32_t r) { return ((float)(r >> 9) + 0.5f) * 1.1920928955078125e-07f; }

// Box-Muller on one word pair: (rho cos(2 pi u1), rho sin(2 pi u1)), rho = sqrt(-2 ln u0).
__device__ __forceinline__ void box_muller(uint32_t r0, uint32_t r1, float& z0, float& z1) {
    const float rho = sqrtf(-2.0f * logf(u01(r0)));
    float s, c;
    sincospif(2.0f * u01(r1), &s, &c);
    z0 = rho * c;
    z1 = rho * s;
}

__device__ __forceinline__ void block_normals(uint64_t block, uint64_t seed, uint64_t step, float z[4]) {
    const u32x4 r = philox_block(block, seed, step);
    box_muller(r.x, r.y, z[0], z[1]);
    box_muller(r.z, r.w, z[2], z[3]);
}

struct AdamArgs {
    float noise_scale;  // sigma * C
    float inv_batch;    // 1 / |B_t|
    float beta1, beta2;
    float inv_bc1, inv_bc2;  // 1 / (1 - beta^t)
    float lr, eps, wd;
};

__device__ __forceinline__ void adam_elem(float& th, float& m, float& v, float s, float z, const AdamArgs& a) {
    const float g = (s + a.noise_scale * z) * a.inv_batch;
    m = a.beta1 * m + (1.0f - a.beta1) * g;
    v = a.beta2 * v + (1.0f - a.beta2) * (g * g);
    const float mh = m * a.inv_bc1;
    const float vh = v * a.inv_bc2;
    th = th - a.lr * (mh / (sqrtf(vh) + a.eps) + a.wd * th);
}

// Gradient signal-to-noise terms (Section 5.2.1): with SNR the kernels also form the squares of the sum and of
// the noise sigma*C*z they read / draw anyway, reduce them over the workgroup in a fixed order and store one
// pair per workgroup at snr_part[2 * (part0 + blockIdx.x)]; snr_finish_kernel adds the pairs in index order.
template <bool SNR>
__device__ __forceinline__ void snr_store(float sig, float noi, float* __restrict__ snr_part, uint64_t slot) {
    if (!SNR) return;
    __shared__ float red[2][4];
    sig = dp_wave_sum(sig);
    noi = dp_wave_sum(noi);
    if ((threadIdx.x & 63) == 0) {
        red[0][threadIdx.x >> 6] = sig;
        red[1][threadIdx.x >> 6] = noi;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        snr_part[2 * slot] = (red[0][0] + red[0][1]) + (red[0][2] + red[0][3]);
        snr_part[2 * slot + 1] = (red[1][0] + red[1][1]) + (red[1][2] + red[1][3]);
    }
}

// Fast path: elem_offset % 4 == 0 and 16-byte aligned pointers.  Thread i owns local elements 4i .. 4i+3.
// Every byte is touched exactly once per step, so loads and stores carry the non-temporal hint (no reuse to keep
// in L2, and lines of the 4 x 1.3 GB state do not evict each other's neighbours).
template <bool NOISE, bool ZERO, bool SNR>
__global__ __launch_bounds__(256) void noise_adamw_vec4(float* __restrict__ params, float* __restrict__ m,
                                                        float* __restrict__ v, float* __restrict__ sum,
                                                        uint64_t nblocks4, uint64_t block0, uint64_t seed,
                                                        uint64_t step, AdamArgs a, float* __restrict__ snr_part) {
    const uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    float sig = 0.f, noi = 0.f;
    if (i < nblocks4) {
        f32x4_t* pt = reinterpret_cast<f32x4_t*>(params) + i;
        f32x4_t* pm = reinterpret_cast<f32x4_t*>(m) + i;
        f32x4_t* pv = reinterpret_cast<f32x4_t*>(v) + i;
        f32x4_t* ps = reinterpret_cast<f32x4_t*>(sum) + i;
        f32x4_t th = __builtin_nontemporal_load(pt);
        f32x4_t mm = __builtin_nontemporal_load(pm);
        f32x4_t vv = __builtin_nontemporal_load(pv);
        const f32x4_t ss = __builtin_nontemporal_load(ps);
        float z[4] = {0.f, 0.f, 0.f, 0.f};
        if (NOISE) block_normals(block0 + i, seed, step, z);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            float t = th[k], mk = mm[k], vk = vv[k];
            adam_elem(t, mk, vk, ss[k], z[k], a);
            th[k] = t;
            mm[k] = mk;
            vv[k] = vk;
        }
        __builtin_nontemporal_store(th, pt);
        __builtin_nontemporal_store(mm, pm);
        __builtin_nontemporal_store(vv, pv);
        if (ZERO) __builtin_nontemporal_store(f32x4_t{0.f, 0.f, 0.f, 0.f}, ps);
        if (SNR) {
            sig = (ss[0] * ss[0] + ss[1] * ss[1]) + (ss[2] * ss[2] + ss[3] * ss[3]);
            const float n0 = a.noise_scale * z[0], n1 = a.noise_scale * z[1], n2 = a.noise_scale * z[2],
                        n3 = a.noise_scale * z[3];
            noi = (n0 * n0 + n1 * n1) + (n2 * n2 + n3 * n3);
        }
    }
    snr_store<SNR>(sig, noi, snr_part, blockIdx.x);
}

// General path: any offset / alignment, and the ragged tail of the fast path.  Thread i owns the Philox
// block first_block + i and touches only those of its four elements that fall inside [e_lo, e_hi).
// `base_elem` is the global index of params[0].
template <bool NOISE, bool ZERO, bool SNR>
__global__ __launch_bounds__(256) void noise_adamw_scalar(float* __restrict__ params, float* __restrict__ m,
                                                          float* __restrict__ v, float* __restrict__ sum,
                                                          uint64_t base_elem, uint64_t e_lo, uint64_t e_hi,
                                                          uint64_t first_block, uint64_t nblocks, uint64_t seed,
                                                          uint64_t step, AdamArgs a, float* __restrict__ snr_part,
                                                          uint64_t part0) {
    const uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    float sig = 0.f, noi = 0.f;
    if (i < nblocks) {
        const uint64_t blk = first_block + i;
        float z[4] = {0.f, 0.f, 0.f, 0.f};
        if (NOISE) block_normals(blk, seed, step, z);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint64_t e = blk * 4 + k;
            if (e >= e_lo && e < e_hi) {
                const uint64_t j = e - base_elem;
                float th = params[j], mm = m[j], vv = v[j];
                const float sj = sum[j];
                adam_elem(th, mm, vv, sj, z[k], a);
                params[j] = th;
                m[j] = mm;
                v[j] = vv;
                if (ZERO) sum[j] = 0.f;
                if (SNR) {
                    const float nz = a.noise_scale * z[k];
                    sig += sj * sj;
                    noi += nz * nz;
                }
            }
        }
    }
    snr_store<SNR>(sig, noi, snr_part, part0 + blockIdx.x);
}

// sq_out[0] += sum of the signal partials, sq_out[1] += sum of the noise partials, each added in fp64 in a fixed
// order (thread t takes pairs t, t + 1024, ...; then a fixed tree over the 1024 threads).  One workgroup.
__global__ __launch_bounds__(1024) void snr_finish_kernel(const float* __restrict__ snr_part, uint64_t npairs,
                                                          float* __restrict__ sq_out) {
    __shared__ double red[2][1024];
    double sig = 0.0, noi = 0.0;
    for (uint64_t k = threadIdx.x; k < npairs; k += 1024) {
        const float2 pr = reinterpret_cast<const float2*>(snr_part)[k];
        sig += (double)pr.x;
        noi += (double)pr.y;
    }
    red[0][threadIdx.x] = sig;
    red[1][threadIdx.x] = noi;
    __syncthreads();
    for (int w = 512; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) {
            red[0][threadIdx.x] += red[0][threadIdx.x + w];
            red[1][threadIdx.x] += red[1][threadIdx.x + w];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        sq_out[0] = (float)((double)sq_out[0] + red[0][0]);
        sq_out[1] = (float)((double)sq_out[1] + red[1][0]);
    }
}

// mode 0: raw words, mode 1: normals
template <int MODE>
__global__ __launch_bounds__(256) void philox_dump(void* __restrict__ out, uint64_t off, uint64_t n,
                                                   uint64_t first_block, uint64_t nblocks, uint64_t seed,
                                                   uint64_t step) {
    const uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= nblocks) return;
    const uint64_t blk = first_block + i;
    uint32_t w[4];
    float z[4];
    if (MODE == 0) {
        const u32x4 r = philox_block(blk, seed, step);
        w[0] = r.x; w[1] = r.y; w[2] = r.z; w[3] = r.w;
    } else {
        block_normals(blk, seed, step, z);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint64_t e = blk * 4 + k;
        if (e >= off && e < off + n) {
            if (MODE == 0) reinterpret_cast<uint32_t*>(out)[e - off] = w[k];
            else reinterpret_cast<float*>(out)[e - off] = z[k];
        }
    }
}

__global__ __launch_bounds__(256) void zero_f32_kernel(float* __restrict__ p, uint64_t n) {
    const uint64_t i = ((uint64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i + 4 <= n && (reinterpret_cast<uintptr_t>(p) & 15) == 0) {
        *reinterpret_cast<float4*>(p + i) = make_float4(0.f, 0.f, 0.f, 0.f);
    } else {
        for (uint64_t k = i; k < n && k < i + 4; ++k) p[k] = 0.f;
    }
}

// sqnorms[i] += partial[i*J + 0] + ... + partial[i*J + J-1], in index order.
__global__ __launch_bounds__(256) void finish_partials_kernel(const float* __restrict__ partial, int B, int J,
                                                              float* __restrict__ sqnorms) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= B) return;
    float t = 0.f;
    for (int j = 0; j < J; ++j) t += partial[(size_t)i * J + j];
    sqnorms[i] += t;
}

__global__ __launch_bounds__(256) void clip_factors_kernel(const float* __restrict__ sqnorms, int B, float C,
                                                           float* __restrict__ c, int* __restrict__ err) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < B) {
        const float ci = dp_clip_factor(sqnorms[i], C);
        c[i] = ci;
        if (ci != ci) atomicOr(err, DP_ERRBIT_NORM);
    }
}

// How a slice [off, off + n) is cut into launches: the 16-byte-aligned body in blocks of four elements (vec4 kernel),
// the rest (or everything, when the slice is not aligned) element by element; one partial pair per workgroup.
struct AdamPlan {
    uint64_t nb4, grid4, done, first, nblocks, grid1;
    uint64_t pairs() const { return grid4 + grid1; }
    bool fits() const { return grid4 <= 0x7FFFFFFFull && grid1 <= 0x7FFFFFFFull; }
};
AdamPlan plan_adamw(const float* params, const float* m, const float* v, const float* sum, uint64_t n, uint64_t off) {
    AdamPlan p{};
    const bool aligned = (off % 4 == 0) && (((uintptr_t)params | (uintptr_t)m | (uintptr_t)v | (uintptr_t)sum) & 15) == 0;
    p.nb4 = (aligned && n >= 4) ? n / 4 : 0;
    p.grid4 = (p.nb4 + 255) / 256;
    p.done = p.nb4 * 4;
    if (p.done < n) {
        p.first = (off + p.done) / 4;
        p.nblocks = (off + n - 1) / 4 - p.first + 1;
        p.grid1 = (p.nblocks + 255) / 256;
    }
    return p;
}

// `part`: room for 2 * plan.pairs() floats when SNR (every pair is overwritten), else unused.  Returns the first
// launch error.
template <bool NOISE, bool ZERO, bool SNR>
hipError_t launch_adamw(hipStream_t stream, const AdamPlan& pl, float* params, float* m, float* v, float* sum, uint64_t n,
                        uint64_t off, uint64_t seed, uint64_t step, const AdamArgs& a, float* part, float* sq_out) {
    hipError_t e = hipSuccess;
    if (pl.grid4) {
        hipLaunchKernelGGL((noise_adamw_vec4<NOISE, ZERO, SNR>), dim3((unsigned)pl.grid4), dim3(256), 0, stream, params, m,
                           v, sum, pl.nb4, off / 4, seed, step, a, part);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if (pl.grid1) {
        hipLaunchKernelGGL((noise_adamw_scalar<NOISE, ZERO, SNR>), dim3((unsigned)pl.grid1), dim3(256), 0, stream, params,
                           m, v, sum, off, off + pl.done, off + n, pl.first, pl.nblocks, seed, step, a, part, pl.grid4);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if (SNR) {
        hipLaunchKernelGGL(snr_finish_kernel, dim3(1), dim3(1024), 0, stream, part, pl.pairs(), sq_out);
        e = hipGetLastError();
    }
    return e;
}

template <bool SNR>
hipError_t dispatch_adamw(hipStream_t stream, const AdamPlan& pl, float* params, float* m, float* v, float* sum, uint64_t n,
                          uint64_t off, uint64_t seed, uint64_t step, const AdamArgs& a, bool noise, int zero_sum,
                          float* part, float* sq_out) {
    if (noise && zero_sum) return launch_adamw<true, true, SNR>(stream, pl, params, m, v, sum, n, off, seed, step, a, part, sq_out);
    if (noise) return launch_adamw<true, false, SNR>(stream, pl, params, m, v, sum, n, off, seed, step, a, part, sq_out);
    if (zero_sum) return launch_adamw<false, true, SNR>(stream, pl, params, m, v, sum, n, off, seed, step, a, part, sq_out);
    return launch_adamw<false, false, SNR>(stream, pl, params, m, v, sum, n, off, seed, step, a, part, sq_out);
}

AdamArgs adam_args(float sigma, float C, uint64_t step, uint64_t batch, float lr, float b1, float b2, float eps, float wd) {
    AdamArgs a;
    a.noise_scale = sigma * C;
    a.inv_batch = (float)(1.0 / (double)batch);
    a.beta1 = b1;
    a.beta2 = b2;
    a.inv_bc1 = (float)(1.0 / (1.0 - pow((double)b1, (double)step)));
    a.inv_bc2 = (float)(1.0 / (1.0 - pow((double)b2, (double)step)));
    a.lr = lr;
    a.eps = eps;
    a.wd = wd;
    return a;
}

}  // namespace

// Device address of dp_static_scratch on the CURRENT device, looked up once per device.
dp_status dpk_static_scratch(float** out) {
    constexpr int MAX_DEV = 64;
    static std::mutex mu;
    static float* ptr[MAX_DEV] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEV) return DP_ERR_HIP;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(dp_static_scratch)) != hipSuccess || !p) return DP_ERR_HIP;
        ptr[dev] = static_cast<float*>(p);
    }
    *out = ptr[dev];
    return DP_OK;
}

// The update with the gradient-SNR terms on `stream`, partial pairs in the static scratch; arguments already checked.
dp_status dpk_noise_adamw_snr_static(hipStream_t stream, float* params, float* m, float* v, float* sum, uint64_t n,
                                     uint64_t off, float sigma, float C, uint64_t seed, uint64_t step, uint64_t batch,
                                     float lr, float b1, float b2, float eps, float wd, int zero_sum, float* sq_out) {
    if (n == 0) return DP_OK;
    if (n > DP_STATIC_MAX_ELEMS) return DP_ERR_WORKSPACE;
    const AdamPlan pl = plan_adamw(params, m, v, sum, n, off);
    if (!pl.fits() || pl.pairs() > DP_STATIC_MAX_PAIRS) return DP_ERR_WORKSPACE;
    float* part = nullptr;
    const dp_status st = dpk_static_scratch(&part);
    if (st != DP_OK) return st;
    const AdamArgs a = adam_args(sigma, C, step, batch, lr, b1, b2, eps, wd);
    const hipError_t e = dispatch_adamw<true>(stream, pl, params, m, v, sum, n, off, seed, step, a, sigma != 0.f, zero_sum,
                                              part, sq_out);
    return e == hipSuccess ? DP_OK : DP_ERR_HIP;
}

dp_status dpk_noise_adamw(dp_ctx* ctx, float* params, float* m, float* v, float* sum, uint64_t n, uint64_t off,
                          float sigma, float C, uint64_t seed, uint64_t step, uint64_t batch, float lr, float b1,
                          float b2, float eps, float wd, int zero_sum, float* sq_out) {
    if (n == 0) return DP_OK;
    const AdamArgs a = adam_args(sigma, C, step, batch, lr, b1, b2, eps, wd);
    const AdamPlan pl = plan_adamw(params, m, v, sum, n, off);
    if (!pl.fits()) {
        DP_SET_ERR(ctx, "dp_noise_adamw: slice too large for one launch");
        return DP_ERR_SHAPE;
    }
    float* part = nullptr;
    if (sq_out) {
        dp_ws_alloc ws(ctx);
        part = ws.get<float>(2 * pl.pairs());
        if (!part) {
            DP_SET_ERR(ctx, "dp_noise_adamw_snr: workspace too small for the per-workgroup partial norms");
            return DP_ERR_WORKSPACE;
        }
    }
    const bool noise = sigma != 0.f;
    dp_prof_scope prof(ctx, DP_PROF_ADAMW, (zero_sum ? 32.0 : 28.0) * (double)n);
    const hipError_t e = sq_out ? dispatch_adamw<true>(ctx->stream, pl, params, m, v, sum, n, off, seed, step, a, noise, zero_sum, part, sq_out)
                                : dispatch_adamw<false>(ctx->stream, pl, params, m, v, sum, n, off, seed, step, a, noise, zero_sum, nullptr, nullptr);
    if (e != hipSuccess) {
        DP_SET_ERR(ctx, "launch of the noise + Adam update failed: %s", hipGetErrorString(e));
        return DP_ERR_HIP;
    }
    return DP_OK;
}

template <int MODE>
static dp_status philox_dump_launch(dp_ctx* ctx, void* out, uint64_t n, uint64_t off, uint64_t seed, uint64_t step) {
    if (n == 0) return DP_OK;
    const uint64_t first = off / 4, last = (off + n - 1) / 4;
    const uint64_t nblocks = last - first + 1;
    const uint64_t grid = (nblocks + 255) / 256;
    if (grid > 0x7FFFFFFFull) {
        DP_SET_ERR(ctx, "philox dump: too many elements for one launch");
        return DP_ERR_SHAPE;
    }
    hipLaunchKernelGGL((philox_dump<MODE>), dim3((unsigned)grid), dim3(256), 0, ctx->stream, out, off, n, first,
                       nblocks, seed, step);
    DP_LAUNCH_CHECK(ctx, "philox_dump");
    return DP_OK;
}

dp_status dpk_philox_u32(dp_ctx* ctx, uint32_t* out, uint64_t n, uint64_t off, uint64_t seed, uint64_t step) {
    return philox_dump_launch<0>(ctx, out, n, off, seed, step);
}
dp_status dpk_normal_f32(dp_ctx* ctx, float* out, uint64_t n, uint64_t off, uint64_t seed, uint64_t step) {
    return philox_dump_launch<1>(ctx, out, n, off, seed, step);
}

dp_status dpk_zero_f32(dp_ctx* ctx, float* p, uint64_t n) {
    if (n == 0) return DP_OK;
    const uint64_t grid = (n + 1023) / 1024;
    if (grid > 0x7FFFFFFFull) {
        DP_SET_ERR(ctx, "dp_zero_f32: too many elements for one launch");
        return DP_ERR_SHAPE;
    }
    hipLaunchKernelGGL(zero_f32_kernel, dim3((unsigned)grid), dim3(256), 0, ctx->stream, p, n);
    DP_LAUNCH_CHECK(ctx, "zero_f32");
    return DP_OK;
}

dp_status dpk_finish_partials(dp_ctx* ctx, const float* partial, int B, int J, float* sqnorms) {
    hipLaunchKernelGGL(finish_partials_kernel, dim3((B + 255) / 256), dim3(256), 0, ctx->stream, partial, B, J,
                       sqnorms);
    DP_LAUNCH_CHECK(ctx, "finish_partials");
    return DP_OK;
}

dp_status dpk_clip_factors(dp_ctx* ctx, const float* sqnorms, int B, float C, float* c) {
    hipLaunchKernelGGL(clip_factors_kernel, dim3((B + 255) / 256), dim3(256), 0, ctx->stream, sqnorms, B, C, c,
                       ctx->err_word);
    DP_LAUNCH_CHECK(ctx, "clip_factors");
    return DP_OK;
}
