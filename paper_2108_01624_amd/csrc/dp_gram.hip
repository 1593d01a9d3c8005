// Per-example squared norm of a dense layer's weight (and bias) gradient from Gram matrices:
//     ||A_i^T G_i||_F^2 = sum_{t,s} (a_t . a_s)(g_t . g_s),      ||sum_t g_t||^2 = sum_{t,s} g_t . g_s
// (the identity follows from the outer-product form of a dense layer's gradient, Section 4.3).
//
// bf16 kernel: one workgroup (4 waves) owns a 128 x 128 block (tb, sb), tb <= sb, of one example's T x T
// plane.  It forms that block of A A^T (contraction over d_in) and of G G^T (over d_out) with
// v_mfma_f32_32x32x16_bf16, both operands being rows of the same tensor with the contraction index
// contiguous in memory (the layout MFMA wants: no transpose anywhere), then multiplies the two
// accumulator sets element by element in registers.  Symmetry halves the work: blocks below the diagonal
// are never launched, and inside a diagonal block the lower-left wave quadrant is skipped while the
// upper-right one counts twice.
//
// Roofline: HBM at T = 128 (2*T*(d_in+d_out) bytes per example against 2*T^2*(d_in+d_out) flops, i.e.
// T flop/B, below the machine balance of ~310 flop/B); each row panel is read once per block it is in.
#include "dp_common.h"

namespace {

constexpr int GB = 128;       // block edge in the (t, s) plane
constexpr int GK = 64;        // contraction chunk staged per step
constexpr int GLD = GK + 8;   // LDS row pitch in bf16 elements (144 B: 16-byte reads of consecutive rows
                              // fall into distinct banks)

struct GramStage {
    uint4 r[4];  // row panel: 4 x 16 B per thread
    uint4 c[4];  // column panel (off-diagonal blocks only)
};

// Load one GK-wide chunk of a 128-row panel of X (rows row0.., all of example `ex`) into registers.
__device__ __forceinline__ void gram_load_panel(const uint16_t* __restrict__ X, size_t ex_base, int row0, int T, int d,
                                                int k0, uint4 v[4]) {
    const int tid = threadIdx.x;
    const int kc = k0 + (tid & 7) * 8;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int row = row0 + (tid >> 3) + 32 * j;
        if (row < T && kc < d)
            v[j] = *reinterpret_cast<const uint4*>(X + ex_base + (size_t)row * d + kc);
        else
            v[j] = make_uint4(0u, 0u, 0u, 0u);
    }
}

__device__ __forceinline__ void gram_store_panel(uint16_t* __restrict__ panel, const uint4 v[4]) {
    const int tid = threadIdx.x;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int row = (tid >> 3) + 32 * j;
        *reinterpret_cast<uint4*>(panel + row * GLD + (tid & 7) * 8) = v[j];
    }
}

__device__ __forceinline__ bf16x8_t gram_frag(const uint16_t* __restrict__ panel, int row, int koff) {
    const uint4 w = *reinterpret_cast<const uint4*>(panel + row * GLD + koff);
    return __builtin_bit_cast(bf16x8_t, w);
}

// Accumulate the (tb, sb) block of X X^T into acc[2][2] (this wave's 64 x 64 quadrant).
template <bool OFFDIAG>
__device__ __forceinline__ void gram_accumulate(const uint16_t* __restrict__ X, size_t ex_base, int T, int d, int tb,
                                                int sb, uint16_t* __restrict__ lds, bool active, int wr, int wc,
                                                f32x16_t acc[2][2]) {
    // LDS layout: [stage][panel(0=row,1=col)][128][GLD]
    constexpr int PANEL = GB * GLD;
    constexpr int STAGE = (OFFDIAG ? 2 : 1) * PANEL;
    const int lane = threadIdx.x & 63;
    const int nch = (d + GK - 1) / GK;
    GramStage st;
    gram_load_panel(X, ex_base, tb * GB, T, d, 0, st.r);
    if (OFFDIAG) gram_load_panel(X, ex_base, sb * GB, T, d, 0, st.c);
    __syncthreads();  // the previous contraction's readers are done with stage 0
    gram_store_panel(lds, st.r);
    if (OFFDIAG) gram_store_panel(lds + PANEL, st.c);
    __syncthreads();
    for (int ch = 0; ch < nch; ++ch) {
        const uint16_t* cur = lds + (ch & 1) * STAGE;
        uint16_t* nxt = lds + ((ch + 1) & 1) * STAGE;
        const bool more = ch + 1 < nch;
        if (more) {
            gram_load_panel(X, ex_base, tb * GB, T, d, (ch + 1) * GK, st.r);
            if (OFFDIAG) gram_load_panel(X, ex_base, sb * GB, T, d, (ch + 1) * GK, st.c);
        }
        if (active) {
            const uint16_t* rp = cur;
            const uint16_t* cp = OFFDIAG ? cur + PANEL : cur;
#pragma unroll
            for (int kk = 0; kk < GK / 16; ++kk) {
                const int koff = kk * 16 + (lane >> 5) * 8;
                bf16x8_t fr[2], fc[2];
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    fr[u] = gram_frag(rp, wr * 64 + u * 32 + (lane & 31), koff);
                    fc[u] = gram_frag(cp, wc * 64 + u * 32 + (lane & 31), koff);
                }
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int nt = 0; nt < 2; ++nt)
                        acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[mt], fc[nt], acc[mt][nt], 0, 0, 0);
            }
        }
        if (more) {
            gram_store_panel(nxt, st.r);
            if (OFFDIAG) gram_store_panel(nxt + PANEL, st.c);
        }
        __syncthreads();
    }
}

template <bool OFFDIAG>
__device__ __forceinline__ float gram_block(const uint16_t* __restrict__ A, const uint16_t* __restrict__ G, int i, int T,
                                            int d_in, int d_out, int tb, int sb, float bias_term, uint16_t* lds) {
    const int wave = threadIdx.x >> 6;
    const int wr = wave >> 1, wc = wave & 1;
    const bool diag = tb == sb;
    const bool active = !(diag && wr > wc);
    const float weight = diag ? (wr == wc ? 1.f : (wr < wc ? 2.f : 0.f)) : 2.f;
    f32x16_t accA[2][2], accG[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) accA[a][b][r] = accG[a][b][r] = 0.f;
    gram_accumulate<OFFDIAG>(A, (size_t)i * T * d_in, T, d_in, tb, sb, lds, active, wr, wc, accA);
    gram_accumulate<OFFDIAG>(G, (size_t)i * T * d_out, T, d_out, tb, sb, lds, active, wr, wc, accG);
    float s = 0.f;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) s += (accA[a][b][r] + bias_term) * accG[a][b][r];
    return s * weight;
}

// grid: npairs == 1: one workgroup per example.  npairs > 1: workgroup id g -> XCD g % 8 (hardware
// round-robin); all block pairs of an example are given ids of one XCD so that the example's row panels,
// each needed by several pairs, are served by that XCD's L2:  example = (g / 8 / npairs) * 8 + g % 8.
__global__ __launch_bounds__(256, 2) void gram_bf16_kernel(const uint16_t* __restrict__ A,
                                                           const uint16_t* __restrict__ G, int B, int T, int d_in,
                                                           int d_out, int has_bias, int nblk, int npairs,
                                                           float* __restrict__ out, int direct) {
    extern __shared__ __attribute__((aligned(16))) uint16_t gram_lds[];
    __shared__ float wred[4];
    int i, pair;
    if (npairs == 1) {
        i = blockIdx.x;
        pair = 0;
    } else {
        const int g = blockIdx.x;
        const int slot = g >> 3;
        i = (slot / npairs) * 8 + (g & 7);
        pair = slot % npairs;
        if (i >= B) return;
    }
    int tb = 0, sb = 0;
    {
        int p = pair;
        while (p >= nblk - tb) {  // row tb of the upper triangle holds nblk - tb pairs
            p -= nblk - tb;
            ++tb;
        }
        sb = tb + p;
    }
    const float bias_term = has_bias ? 1.f : 0.f;
    float s;
    if (tb == sb) s = gram_block<false>(A, G, i, T, d_in, d_out, tb, sb, bias_term, gram_lds);
    else s = gram_block<true>(A, G, i, T, d_in, d_out, tb, sb, bias_term, gram_lds);
    const float tot = dp_block_sum<256>(s, wred);
    if (threadIdx.x == 0) {
        if (direct) out[i] += tot;
        else out[(size_t)i * npairs + pair] = tot;
    }
}

// fp32 reference-precision paths (small shapes; parity configuration with fp32 inputs).
// One workgroup per example; thread-strided loop over the pairs t <= s.
__global__ __launch_bounds__(256) void gram_f32_kernel(const float* __restrict__ A, const float* __restrict__ G, int T,
                                                       int d_in, int d_out, int has_bias, float* __restrict__ out) {
    __shared__ float wred[4];
    const int i = blockIdx.x;
    const float* Ai = A + (size_t)i * T * d_in;
    const float* Gi = G + (size_t)i * T * d_out;
    const long npairs = (long)T * (T + 1) / 2;
    float s = 0.f;
    for (long p = threadIdx.x; p < npairs; p += 256) {
        // invert p = t*T - t(t-1)/2 + (s - t)
        int t = 0;
        long q = p;
        while (q >= T - t) {
            q -= T - t;
            ++t;
        }
        const int u = t + (int)q;
        float aa = 0.f, gg = 0.f;
        for (int k = 0; k < d_in; ++k) aa += Ai[(size_t)t * d_in + k] * Ai[(size_t)u * d_in + k];
        for (int k = 0; k < d_out; ++k) gg += Gi[(size_t)t * d_out + k] * Gi[(size_t)u * d_out + k];
        const float w = t == u ? 1.f : 2.f;
        s += w * (aa + (has_bias ? 1.f : 0.f)) * gg;
    }
    const float tot = dp_block_sum<256>(s, wred);
    if (threadIdx.x == 0) out[i] += tot;
}

// fp32 materialise: every entry of A_i^T G_i is formed and squared.
__global__ __launch_bounds__(256) void materialise_f32_kernel(const float* __restrict__ A, const float* __restrict__ G,
                                                              int T, int d_in, int d_out, float* __restrict__ out) {
    __shared__ float wred[4];
    const int i = blockIdx.x;
    const float* Ai = A + (size_t)i * T * d_in;
    const float* Gi = G + (size_t)i * T * d_out;
    const long n = (long)d_in * d_out;
    float s = 0.f;
    for (long e = threadIdx.x; e < n; e += 256) {
        const int p = (int)(e / d_out), q = (int)(e % d_out);
        float acc = 0.f;
        for (int t = 0; t < T; ++t) acc += Ai[(size_t)t * d_in + p] * Gi[(size_t)t * d_out + q];
        s += acc * acc;
    }
    const float tot = dp_block_sum<256>(s, wred);
    if (threadIdx.x == 0) out[i] += tot;
}

}  // namespace

dp_status dpk_gram_sqnorms(dp_ctx* ctx, const void* A, const void* G, dp_dtype dt, int B, int T, int d_in, int d_out,
                           int has_bias, float* sqnorms) {
    if (dt == DP_F32) {
        hipLaunchKernelGGL(gram_f32_kernel, dim3(B), dim3(256), 0, ctx->stream, (const float*)A, (const float*)G, T,
                           d_in, d_out, has_bias, sqnorms);
        DP_LAUNCH_CHECK(ctx, "gram_f32");
        return DP_OK;
    }
    const int nblk = (T + GB - 1) / GB;
    const long npairs = (long)nblk * (nblk + 1) / 2;
    const size_t lds = (size_t)2 * (nblk > 1 ? 2 : 1) * GB * GLD * sizeof(uint16_t);
    static bool lds_attr_set = false;  // off-diagonal blocks stage two panels per step: 72 KiB of dynamic LDS
    if (!lds_attr_set) {
        DP_HIP_CHECK(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(gram_bf16_kernel),
                                              hipFuncAttributeMaxDynamicSharedMemorySize,
                                              2 * 2 * GB * GLD * (int)sizeof(uint16_t)));
        lds_attr_set = true;
    }
    const double bytes = 2.0 * (double)B * T * ((double)d_in + d_out);
    if (npairs == 1) {
        dp_prof_scope prof(ctx, DP_PROF_GRAM, bytes);
        hipLaunchKernelGGL(gram_bf16_kernel, dim3(B), dim3(256), lds, ctx->stream, (const uint16_t*)A,
                           (const uint16_t*)G, B, T, d_in, d_out, has_bias, nblk, 1, sqnorms, 1);
        DP_LAUNCH_CHECK(ctx, "gram_bf16");
        return DP_OK;
    }
    const long groups = (B + 7) / 8;
    const long nwg = groups * 8 * npairs;
    if (nwg > 0x7FFFFFFFl) {
        DP_SET_ERR(ctx, "dp_sqnorms_dense: B * T^2 too large for one launch");
        return DP_ERR_SHAPE;
    }
    dp_ws_alloc ws(ctx);
    float* part = ws.get<float>((size_t)B * npairs);
    if (!part) {
        DP_SET_ERR(ctx, "workspace too small for %d x %ld Gram partials", B, npairs);
        return DP_ERR_WORKSPACE;
    }
    {
        dp_prof_scope prof(ctx, DP_PROF_GRAM, bytes);
        hipLaunchKernelGGL(gram_bf16_kernel, dim3((unsigned)nwg), dim3(256), lds, ctx->stream, (const uint16_t*)A,
                           (const uint16_t*)G, B, T, d_in, d_out, has_bias, nblk, (int)npairs, part, 0);
    }
    DP_LAUNCH_CHECK(ctx, "gram_bf16");
    return dpk_finish_partials(ctx, part, B, (int)npairs, sqnorms);
}

dp_status dpk_materialise_f32(dp_ctx* ctx, const float* A, const float* G, int B, int T, int d_in, int d_out,
                              float* sqnorms) {
    hipLaunchKernelGGL(materialise_f32_kernel, dim3(B), dim3(256), 0, ctx->stream, A, G, T, d_in, d_out, sqnorms);
    DP_LAUNCH_CHECK(ctx, "materialise_f32");
    return DP_OK;
}
