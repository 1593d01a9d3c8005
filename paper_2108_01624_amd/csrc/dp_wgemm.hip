// Clip-weighted dense gradient sum  S_W += sum_i c_i A_i^T G_i = A_flat^T diag(c (x) 1_T) G_flat
// (the sum over the batch of clip(grad, C) in the g_t line of Algorithm 1, for a dense layer whose
// per-example gradient is the outer-product form of Section 4.3), and the tile-by-tile materialisation
// of one example's A_i^T G_i for the squared-norm path that sums squares of the entries.
//
// Both are "TN" contractions: the contraction index (token row k) is the SLOW index of both operands in
// memory, while v_mfma_f32_32x32x16_bf16 wants each lane to hold 8 consecutive k for one output row/column.
// The kernel stages [k][p] tiles in LDS exactly as they lie in memory (16-byte coalesced global loads,
// 16-byte LDS stores), and each lane then reads, for 8 consecutive k rows, the MI (NI) adjacent columns it
// owns (one 8-byte LDS read per row when MI = 4) and regroups them with v_perm_b32 into MI fragments.
// Lane m of fragment j therefore holds column  MI*m + j  of the wave tile: the MFMA row index is a
// permutation of the tile's columns, undone for free in the epilogue, where a lane ends up with NI
// consecutive output columns per row and stores them as one 16-byte vector.
//
// The clip factor c_i multiplies the rows of G in fp32 while the tile is staged (once per element per
// workgroup) and the product is rounded to bf16 (nearest even); accumulation is fp32 in the MFMA.
//
// Roofline: MFMA.  2*B*T*d_in*d_out flops per layer against (d_in + d_out)*B*T*2 bytes read once.
#include "dp_common.h"

namespace {

constexpr int BK = 32;  // token rows per staged tile

enum { EPI_STORE = 0, EPI_ADD = 1, EPI_SQNORM = 2 };

struct WgemmArgs {
    const uint16_t* A;   // [K, d_in]
    const uint16_t* G;   // [K, d_out]
    const float* c;      // [B] clip factors (nullptr: weight 1)
    int T, d_in, d_out;
    long K;              // total rows
    long rows_per_split; // multiple of BK
    int tiles_m, tiles_n, nsplit;
    float* out;          // EPI_STORE: [nsplit][d_in][d_out]; EPI_ADD: [d_in][d_out]; EPI_SQNORM: [nsplit][ntiles]
    int xcd_map;         // 1: split index interleaved over the 8 XCDs
};

__device__ __forceinline__ uint32_t perm_lo(uint32_t hi_src, uint32_t lo_src) {
    return __builtin_amdgcn_perm(hi_src, lo_src, 0x05040100u);  // [lo_src.lo16, hi_src.lo16]
}
__device__ __forceinline__ uint32_t perm_hi(uint32_t hi_src, uint32_t lo_src) {
    return __builtin_amdgcn_perm(hi_src, lo_src, 0x07060302u);  // [lo_src.hi16, hi_src.hi16]
}

template <int NV>
struct RawRow;  // NV 32-bit words = 2*NV adjacent bf16 columns of one k row
template <>
struct RawRow<1> {
    uint32_t w[1];
    __device__ __forceinline__ void load(const uint16_t* p) { w[0] = *reinterpret_cast<const uint32_t*>(p); }
};
template <>
struct RawRow<2> {
    uint32_t w[2];
    __device__ __forceinline__ void load(const uint16_t* p) {
        const uint2 v = *reinterpret_cast<const uint2*>(p);
        w[0] = v.x;
        w[1] = v.y;
    }
};

// Build the NF (= 2 or 4) MFMA fragments of one operand for one 16-row k step.
// tile: LDS tile [BK][LD]; col0: first of this lane's NF adjacent columns; krow0: first of its 8 k rows.
template <int NF, int LD>
__device__ __forceinline__ void build_frags(const uint16_t* __restrict__ tile, int col0, int krow0, bf16x8_t frag[NF]) {
    RawRow<NF / 2> raw[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) raw[e].load(tile + (krow0 + e) * LD + col0);
#pragma unroll
    for (int j2 = 0; j2 < NF / 2; ++j2) {
        uint32_t lo[4], hi[4];
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
            lo[e2] = perm_lo(raw[2 * e2 + 1].w[j2], raw[2 * e2].w[j2]);
            hi[e2] = perm_hi(raw[2 * e2 + 1].w[j2], raw[2 * e2].w[j2]);
        }
        frag[2 * j2] = __builtin_bit_cast(bf16x8_t, make_uint4(lo[0], lo[1], lo[2], lo[3]));
        frag[2 * j2 + 1] = __builtin_bit_cast(bf16x8_t, make_uint4(hi[0], hi[1], hi[2], hi[3]));
    }
}

__device__ __forceinline__ uint4 scale_bf16x8(uint4 v, float s) {
    uint4 o;
    o.x = dp_pack_bf16x2(dp_bf16_lo(v.x) * s, dp_bf16_hi(v.x) * s);
    o.y = dp_pack_bf16x2(dp_bf16_lo(v.y) * s, dp_bf16_hi(v.y) * s);
    o.z = dp_pack_bf16x2(dp_bf16_lo(v.z) * s, dp_bf16_hi(v.z) * s);
    o.w = dp_pack_bf16x2(dp_bf16_lo(v.w) * s, dp_bf16_hi(v.w) * s);
    return o;
}

// Workgroup = 4 waves as 2 x 2; wave tile (32*MI) x (32*NI); block tile BM x BN = (64*MI) x (64*NI).
template <int MI, int NI, int EPI>
__global__ __launch_bounds__(256) void wgemm_bf16_kernel(WgemmArgs a) {
    constexpr int BM = 64 * MI, BN = 64 * NI;
    constexpr int WM = 32 * MI, WN = 32 * NI;
    constexpr int LDA = BM + 8, LDG = BN + 8;  // bf16 elements; +16 B keeps 16-byte alignment of every row
    __shared__ __attribute__((aligned(16))) uint16_t As[2][BK * LDA];
    __shared__ __attribute__((aligned(16))) uint16_t Gs[2][BK * LDG];
    __shared__ float wred[4];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wr = wave >> 1, wc = wave & 1;
    const int ntiles = a.tiles_m * a.tiles_n;
    int tile, split;
    if (a.xcd_map) {
        const int g = blockIdx.x, slot = g >> 3;
        split = (slot / ntiles) * 8 + (g & 7);
        tile = slot % ntiles;
        if (split >= a.nsplit) return;
    } else {
        tile = blockIdx.x % ntiles;
        split = blockIdx.x / ntiles;
    }
    const int pm = tile / a.tiles_n, qn = tile % a.tiles_n;
    const int p0 = pm * BM, q0 = qn * BN;
    const long k_lo = (long)split * a.rows_per_split;
    const long k_hi = k_lo + a.rows_per_split < a.K ? k_lo + a.rows_per_split : a.K;
    const int nsteps = k_hi > k_lo ? (int)((k_hi - k_lo + BK - 1) / BK) : 0;

    f32x16_t acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    uint4 ra[MI], rg[NI];
    auto gload = [&](long kbase) {
#pragma unroll
        for (int j = 0; j < MI; ++j) {
            const int id = tid + 256 * j;
            const int row = id / (BM / 8), cc = (id % (BM / 8)) * 8;
            const long k = kbase + row;
            if (k < k_hi && p0 + cc < a.d_in)
                ra[j] = *reinterpret_cast<const uint4*>(a.A + (size_t)k * a.d_in + p0 + cc);
            else
                ra[j] = make_uint4(0u, 0u, 0u, 0u);
        }
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const int id = tid + 256 * j;
            const int row = id / (BN / 8), cc = (id % (BN / 8)) * 8;
            const long k = kbase + row;
            if (k < k_hi && q0 + cc < a.d_out) {
                const uint4 v = *reinterpret_cast<const uint4*>(a.G + (size_t)k * a.d_out + q0 + cc);
                rg[j] = a.c ? scale_bf16x8(v, a.c[(uint32_t)k / (uint32_t)a.T]) : v;
            } else {
                rg[j] = make_uint4(0u, 0u, 0u, 0u);
            }
        }
    };
    auto lstore = [&](int stage) {
#pragma unroll
        for (int j = 0; j < MI; ++j) {
            const int id = tid + 256 * j;
            const int row = id / (BM / 8), cc = (id % (BM / 8)) * 8;
            *reinterpret_cast<uint4*>(&As[stage][row * LDA + cc]) = ra[j];
        }
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const int id = tid + 256 * j;
            const int row = id / (BN / 8), cc = (id % (BN / 8)) * 8;
            *reinterpret_cast<uint4*>(&Gs[stage][row * LDG + cc]) = rg[j];
        }
    };

    if (nsteps > 0) {
        gload(k_lo);
        lstore(0);
    }
    __syncthreads();
    for (int s = 0; s < nsteps; ++s) {
        const int cur = s & 1;
        const bool more = s + 1 < nsteps;
        if (more) gload(k_lo + (long)(s + 1) * BK);
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            const int krow0 = kk * 16 + (lane >> 5) * 8;
            bf16x8_t fa[MI], fg[NI];
            build_frags<MI, LDA>(As[cur], wr * WM + MI * (lane & 31), krow0, fa);
            build_frags<NI, LDG>(Gs[cur], wc * WN + NI * (lane & 31), krow0, fg);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fg[j], acc[i][j], 0, 0, 0);
        }
        if (more) lstore(cur ^ 1);
        __syncthreads();
    }

    if (EPI == EPI_SQNORM) {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) s += acc[i][j][r] * acc[i][j][r];
        const float tot = dp_block_sum<256>(s, wred);
        if (tid == 0) a.out[(size_t)split * ntiles + tile] = tot;
        return;
    }

    // MFMA tile (i, j), accumulator register r of lane l holds output row m = 8*(r/4) + 4*(l/32) + r%4 and
    // column n = l%32 of that tile, i.e. p = p0 + wr*WM + MI*m + i and q = q0 + wc*WN + NI*n + j.
    float* base = a.out + (EPI == EPI_STORE ? (size_t)split * a.d_in * a.d_out : (size_t)0);
    const int qcol = q0 + wc * WN + NI * (lane & 31);
    if (qcol < a.d_out) {  // d_out % 8 == 0 and NI divides 8: a lane's NI columns are all in or all out
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                const int p = p0 + wr * WM + MI * m + i;
                if (p < a.d_in) {
                    float* dst = base + (size_t)p * a.d_out + qcol;
                    if constexpr (NI == 4) {
                        float4 v = make_float4(acc[i][0][r], acc[i][1][r], acc[i][2][r], acc[i][3][r]);
                        if (EPI == EPI_ADD) {
                            const float4 o = *reinterpret_cast<const float4*>(dst);
                            v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w;
                        }
                        *reinterpret_cast<float4*>(dst) = v;
                    } else {
                        float2 v = make_float2(acc[i][0][r], acc[i][1][r]);
                        if (EPI == EPI_ADD) {
                            const float2 o = *reinterpret_cast<const float2*>(dst);
                            v.x += o.x; v.y += o.y;
                        }
                        *reinterpret_cast<float2*>(dst) = v;
                    }
                }
            }
    }
}

// ------------------------------------------------------------------------------------------------
// fp32 path (small shapes, fp32 inputs): 64 x 64 output tile per workgroup, 16 x 16 threads, 4 x 4 each.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void wgemm_f32_kernel(const float* __restrict__ A, const float* __restrict__ G,
                                                        const float* __restrict__ c, int T, long K, int d_in,
                                                        int d_out, float* __restrict__ out) {
    __shared__ float As[16][64 + 4];
    __shared__ float Gs[16][64 + 4];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int p0 = blockIdx.y * 64, q0 = blockIdx.x * 64;
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
    for (long k0 = 0; k0 < K; k0 += 16) {
        for (int e = threadIdx.x; e < 16 * 64; e += 256) {
            const int r = e >> 6, col = e & 63;
            const long k = k0 + r;
            const bool ok = k < K;
            As[r][col] = (ok && p0 + col < d_in) ? A[(size_t)k * d_in + p0 + col] : 0.f;
            Gs[r][col] = (ok && q0 + col < d_out) ? c[k / T] * G[(size_t)k * d_out + q0 + col] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float av[4], gv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) av[i] = As[r][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) gv[j] = Gs[r][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] += av[i] * gv[j];
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int p = p0 + ty * 4 + i, q = q0 + tx * 4 + j;
            if (p < d_in && q < d_out) out[(size_t)p * d_out + q] += acc[i][j];
        }
}

template <int MI, int NI, int EPI>
void wgemm_launch(dp_ctx* ctx, const WgemmArgs& a, unsigned grid) {
    hipLaunchKernelGGL((wgemm_bf16_kernel<MI, NI, EPI>), dim3(grid), dim3(256), 0, ctx->stream, a);
}

}  // namespace

// Tile shape: 256 x 256 when both dimensions are at least that large, otherwise 128 x 128.
static inline bool big_tile(int d_in, int d_out) { return d_in >= 256 && d_out >= 256; }

dp_status dpk_weighted_gemm(dp_ctx* ctx, const void* A, const void* G, dp_dtype dt, int B, int T, int d_in, int d_out,
                            const float* c, float* sum_W) {
    const long K = (long)B * T;
    if (dt == DP_F32) {
        dim3 grid((d_out + 63) / 64, (d_in + 63) / 64);
        hipLaunchKernelGGL(wgemm_f32_kernel, grid, dim3(256), 0, ctx->stream, (const float*)A, (const float*)G, c, T, K,
                           d_in, d_out, sum_W);
        DP_LAUNCH_CHECK(ctx, "wgemm_f32");
        return DP_OK;
    }
    const bool big = big_tile(d_in, d_out);
    const int BM = big ? 256 : 128, BN = BM;
    WgemmArgs a;
    a.A = (const uint16_t*)A;
    a.G = (const uint16_t*)G;
    a.c = c;
    a.T = T;
    a.d_in = d_in;
    a.d_out = d_out;
    a.K = K;
    a.tiles_m = (d_in + BM - 1) / BM;
    a.tiles_n = (d_out + BN - 1) / BN;
    const int ntiles = a.tiles_m * a.tiles_n;
    // split the token rows so that about 256 workgroups exist (one per CU: the 256 x 256 tile's accumulators
    // leave room for one workgroup per CU); splits come in multiples of 8 (one per XCD) once there are
    // several, and each split keeps at least 256 rows.
    const long ksteps = (K + BK - 1) / BK;
    long nsplit = 1;
    if (ntiles < 256) {
        nsplit = (256 + ntiles - 1) / ntiles;
        const long max_split = (ksteps + 7) / 8;
        if (nsplit > max_split) nsplit = max_split;
        if (nsplit >= 8) nsplit = (nsplit / 8) * 8;
        if (nsplit < 1) nsplit = 1;
    }
    dp_ws_alloc ws(ctx);
    float* part = nullptr;
    while (nsplit > 1) {
        part = ws.get<float>((size_t)nsplit * d_in * d_out);
        if (part) break;
        nsplit = nsplit > 8 ? nsplit - 8 : nsplit / 2;  // shrink to what the workspace holds
    }
    const long steps_per = (ksteps + nsplit - 1) / nsplit;
    a.rows_per_split = steps_per * BK;
    nsplit = (ksteps + steps_per - 1) / steps_per;
    a.nsplit = (int)nsplit;
    a.xcd_map = nsplit >= 8 ? 1 : 0;
    const long nwg = a.xcd_map ? ((nsplit + 7) / 8) * 8 * ntiles : nsplit * ntiles;
    if (nwg > 0x7FFFFFFFl) {
        DP_SET_ERR(ctx, "dp_clip_accumulate_dense: too many tiles");
        return DP_ERR_SHAPE;
    }
    if (nsplit == 1) {
        a.out = sum_W;
        if (big) wgemm_launch<4, 4, EPI_ADD>(ctx, a, (unsigned)nwg);
        else wgemm_launch<2, 2, EPI_ADD>(ctx, a, (unsigned)nwg);
        DP_LAUNCH_CHECK(ctx, "wgemm_bf16");
        return DP_OK;
    }
    a.out = part;
    if (big) wgemm_launch<4, 4, EPI_STORE>(ctx, a, (unsigned)nwg);
    else wgemm_launch<2, 2, EPI_STORE>(ctx, a, (unsigned)nwg);
    DP_LAUNCH_CHECK(ctx, "wgemm_bf16");
    return dpk_reduce_partials(ctx, part, (int)nsplit, (size_t)d_in * d_out, (size_t)d_in * d_out, sum_W);
}

dp_status dpk_materialise_sqnorms(dp_ctx* ctx, const void* A, const void* G, dp_dtype dt, int B, int T, int d_in,
                                  int d_out, int has_bias, float* sqnorms) {
    dp_status st;
    if (dt == DP_F32) {
        st = dpk_materialise_f32(ctx, (const float*)A, (const float*)G, B, T, d_in, d_out, sqnorms);
    } else {
        const bool big = big_tile(d_in, d_out);
        const int BM = big ? 256 : 128, BN = BM;
        WgemmArgs a;
        a.A = (const uint16_t*)A;
        a.G = (const uint16_t*)G;
        a.c = nullptr;
        a.T = T;
        a.d_in = d_in;
        a.d_out = d_out;
        a.K = (long)B * T;
        a.tiles_m = (d_in + BM - 1) / BM;
        a.tiles_n = (d_out + BN - 1) / BN;
        a.nsplit = B;  // one "split" per example: rows [i*T, (i+1)*T)
        a.rows_per_split = T;
        a.xcd_map = 0;
        const int ntiles = a.tiles_m * a.tiles_n;
        const long nwg = (long)B * ntiles;
        if (nwg > 0x7FFFFFFFl) {
            DP_SET_ERR(ctx, "dp_sqnorms_dense: too many tiles");
            return DP_ERR_SHAPE;
        }
        dp_ws_alloc ws(ctx);
        float* part = ws.get<float>((size_t)B * ntiles);
        if (!part) {
            DP_SET_ERR(ctx, "workspace too small for %d x %d materialise partials", B, ntiles);
            return DP_ERR_WORKSPACE;
        }
        a.out = part;
        if (big) wgemm_launch<4, 4, EPI_SQNORM>(ctx, a, (unsigned)nwg);
        else wgemm_launch<2, 2, EPI_SQNORM>(ctx, a, (unsigned)nwg);
        DP_LAUNCH_CHECK(ctx, "wgemm_bf16 (materialise)");
        st = dpk_finish_partials(ctx, part, B, ntiles, sqnorms);
    }
    if (st != DP_OK) return st;
    if (has_bias) return dpk_colstat_sqnorms(ctx, nullptr, G, dt, B, T, d_out, 0, 1, sqnorms);
    return DP_OK;
}
