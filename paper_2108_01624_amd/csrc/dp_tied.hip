// A table E [V, d] that an example uses twice: as the lookup y_t = E[ids_t] and as the output projection
// logits = H E^T of M selected positions (Section 4.3 names the word-piece table; the tied output projection is
// the usual BERT head, on which the paper is silent).  E is one parameter with one per-example gradient
//     g_i = scatter(ids_i, dY_i) + dL_i^T H_i,
// so  ||g_i||^2 = ||scatter||^2 + ||dL_i^T H_i||^2 + 2 <scatter, dL_i^T H_i>.
// The first two terms are the embedding and the dense norm (kernels of their own); this file holds the third:
//     <scatter, dL_i^T H_i> = sum_t sum_m dL_i[m, ids_t] * <dY_i[t,:], H_i[m,:]>,
// i.e. the T x M matrix P = dY_i H_i^T (a contraction over d, on MFMA for bf16) multiplied element-wise by the
// T x M entries of dL_i gathered at the example's own token ids, summed.
//
// Roofline: HBM, B*(T+M)*d*E bytes read once plus B*T*M gathered elements (each its own 32-byte sector of dL);
// 2*T*M*d flops per example are far below the machine balance.
#include <stdlib.h>

#include "dp_common.h"

namespace {

// bf16: one workgroup (4 waves) per example; a wave owns 32 x 32 tiles (tb, mb) of P.  Operand fragments come
// straight from global memory: lane (row = lane % 32, half = lane / 32) reads 64 contiguous bytes of its row per
// 64-wide chunk of d, so that the two lanes of a row use a whole 128-byte line.  MFMA j of a chunk contracts the
// 16 columns {chunk + half*32 + j*8 + 0..7}: the assignment of columns to the instruction's k slots is the
// same for both operands, which is all a dot product needs.
__global__ __launch_bounds__(256) void tied_cross_bf16_kernel(const int32_t* __restrict__ ids,
                                                              const uint16_t* __restrict__ dY,
                                                              const uint16_t* __restrict__ H,
                                                              const uint16_t* __restrict__ dL, int T, int M, int d, int V,
                                                              float* __restrict__ sqnorms, int* __restrict__ err) {
    __shared__ float red[4];
    const int i = blockIdx.x;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int half = lane >> 5, r32 = lane & 31;
    const int ntb = (T + 31) / 32, nmb = (M + 31) / 32;
    float tot = 0.f;
    bool bad = false;
    for (int tile = wave; tile < ntb * nmb; tile += 4) {
        const int tb = tile / nmb, mb = tile - tb * nmb;
        const int row_t = tb * 32 + r32, row_m = mb * 32 + r32;
        const bool va = row_t < T, vb = row_m < M;
        const uint16_t* pa = dY + ((size_t)i * T + (va ? row_t : 0)) * d;
        const uint16_t* pb = H + ((size_t)i * M + (vb ? row_m : 0)) * d;
        f32x16_t acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
        for (int kb = 0; kb < d; kb += 64) {
            uint4 fa[4], fb[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int k = kb + half * 32 + j * 8;  // d is a multiple of 8: a fragment is inside the row or not at all
                fa[j] = (va && k < d) ? *reinterpret_cast<const uint4*>(pa + k) : make_uint4(0u, 0u, 0u, 0u);
                fb[j] = (vb && k < d) ? *reinterpret_cast<const uint4*>(pb + k) : make_uint4(0u, 0u, 0u, 0u);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, fa[j]),
                                                              __builtin_bit_cast(bf16x8_t, fb[j]), acc, 0, 0, 0);
        }
        // acc[r] of this lane = P[t, m] with t = tb*32 + 8*(r/4) + 4*half + r%4 and m = mb*32 + lane%32
        if (vb) {
            const uint16_t* prow = dL + ((size_t)i * M + row_m) * V;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int t = tb * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
                if (t < T) {
                    const int32_t id = ids[(size_t)i * T + t];
                    if (id >= 0 && id < V) tot += acc[r] * dp_bf16_bits_to_f32(prow[id]);
                    else bad = true;
                }
            }
        }
    }
    if (bad) atomicOr(err, 1);
    tot = dp_block_sum<256>(tot, red);
    if (threadIdx.x == 0) sqnorms[i] += 2.f * tot;
}

// fp32 (correctness path, not tuned): one workgroup per example; lane l keeps
// sum_{t,m} dL[m, ids_t] * sum_{k = l mod 64} dY[t,k] H[m,k], so that one reduction at the end is enough.
__global__ __launch_bounds__(256) void tied_cross_f32_kernel(const int32_t* __restrict__ ids, const float* __restrict__ dY,
                                                             const float* __restrict__ H, const float* __restrict__ dL,
                                                             int T, int M, int d, int V, float* __restrict__ sqnorms,
                                                             int* __restrict__ err) {
    __shared__ float red[4];
    const int i = blockIdx.x;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    float tot = 0.f;
    bool bad = false;
    for (int t = wave; t < T; t += 4) {
        const int32_t id = ids[(size_t)i * T + t];
        if (id < 0 || id >= V) {
            bad = true;
            continue;
        }
        const float* y = dY + ((size_t)i * T + t) * d;
        for (int m = 0; m < M; ++m) {
            const float* h = H + ((size_t)i * M + m) * d;
            float p = 0.f;
            for (int k = lane; k < d; k += 64) p += y[k] * h[k];
            tot += dL[((size_t)i * M + m) * V + id] * p;
        }
    }
    if (bad) atomicOr(err, 1);
    tot = dp_block_sum<256>(tot, red);
    if (threadIdx.x == 0) sqnorms[i] += 2.f * tot;
}

// Hs[i, :] = bf16(c_i * H[i, :]) (round to nearest even), rows of `row_len` elements, 8 elements per thread.
__global__ __launch_bounds__(256) void scale_rows_bf16_kernel(const uint16_t* __restrict__ H, const float* __restrict__ c,
                                                              size_t n8, int row_len8, uint16_t* __restrict__ Hs) {
    const size_t j = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= n8) return;
    const float ci = c[j / row_len8];
    const uint4 w = *reinterpret_cast<const uint4*>(H + j * 8);
    uint4 o;
    o.x = dp_pack_bf16x2(ci * dp_bf16_lo(w.x), ci * dp_bf16_hi(w.x));
    o.y = dp_pack_bf16x2(ci * dp_bf16_lo(w.y), ci * dp_bf16_hi(w.y));
    o.z = dp_pack_bf16x2(ci * dp_bf16_lo(w.z), ci * dp_bf16_hi(w.z));
    o.w = dp_pack_bf16x2(ci * dp_bf16_lo(w.w), ci * dp_bf16_hi(w.w));
    *reinterpret_cast<uint4*>(Hs + j * 8) = o;
}

}  // namespace

// The output projection's sum is a dense sum with input dL [B, M, V] and output gradient H [B, M, d].  M (20 or 80
// prediction slots) is not a multiple of the fast GEMM's 64-row example granularity, but H is small: its rows are
// multiplied by c_i once (rounded to bf16, which is what the general GEMM does with every element it stages), and
// the B*M rows are then contracted as B*M/64 blocks of 64 rows with factor 1 by the fast kernel.
dp_status dpk_tied_projection_sums(dp_ctx* ctx, const void* H, const void* dL, dp_dtype dt, int B, int M, int d, int V,
                                   const float* sqnorms, float C, float* sum_E) {
    const long rows = (long)B * M;
    if (dt == DP_BF16 && rows % 64 == 0 && M % 64 != 0 && V >= 256 && d >= 256 && rows / 64 <= ctx->cbuf_cap) {
        dp_ws_alloc ws(ctx);
        uint16_t* Hs = ws.get<uint16_t>((size_t)rows * d);
        float* zero = ws.get<float>((size_t)(rows / 64));
        if (Hs && zero) {
            dp_status st = dpk_clip_factors(ctx, sqnorms, B, C, ctx->cbuf);
            if (st != DP_OK) return st;
            const size_t n8 = (size_t)rows * d / 8;
            hipLaunchKernelGGL(scale_rows_bf16_kernel, dim3((unsigned)((n8 + 255) / 256)), dim3(256), 0, ctx->stream,
                               (const uint16_t*)H, ctx->cbuf, n8, M * d / 8, Hs);
            DP_LAUNCH_CHECK(ctx, "scale_rows_bf16");
            st = dpk_zero_f32(ctx, zero, (uint64_t)(rows / 64));  // squared norm 0 -> factor 1 for every block of rows
            if (st != DP_OK) return st;
            dp_ws_hold hold(ws);
            return dpk_weighted_gemm(ctx, dL, Hs, dt, (int)(rows / 64), 64, V, d, zero, C, sum_E, nullptr);
        }
    }
    return dpk_weighted_gemm(ctx, dL, H, dt, B, M, V, d, sqnorms, C, sum_E, nullptr);
}

// sqnorms[i] += 2 * sum_{t,m} dL[i,m,ids[i,t]] * <dY[i,t,:], H[i,m,:]>
dp_status dpk_tied_cross_sqnorms(dp_ctx* ctx, const int32_t* ids, const void* dY, const void* H, const void* dL,
                                 dp_dtype dt, int B, int T, int M, int d, int V, float* sqnorms) {
    if (B == 0 || T == 0 || M == 0 || d == 0) return DP_OK;
    if (dt == DP_BF16)
        hipLaunchKernelGGL(tied_cross_bf16_kernel, dim3(B), dim3(256), 0, ctx->stream, ids, (const uint16_t*)dY,
                           (const uint16_t*)H, (const uint16_t*)dL, T, M, d, V, sqnorms, ctx->err_word);
    else
        hipLaunchKernelGGL(tied_cross_f32_kernel, dim3(B), dim3(256), 0, ctx->stream, ids, (const float*)dY,
                           (const float*)H, (const float*)dL, T, M, d, V, sqnorms, ctx->err_word);
    DP_LAUNCH_CHECK(ctx, "tied_cross");
    return DP_OK;
}
