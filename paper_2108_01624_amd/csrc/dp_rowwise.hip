// HBM-bound streaming kernels of the hot path: column statistics (LayerNorm gain/offset and dense-bias
// gradients), embedding-table gradients (per-example segment reduction for the norms, stable radix sort
// plus ordered segment sums for the clip-weighted scatter), and the ordered reduction of partial buffers.
//
// Roofline: HBM.  Each kernel reads its bf16 (or fp32) inputs exactly once; algorithmic bytes per
// example are T*d*elem for every tensor read.  Threads own 4 consecutive columns (8-byte bf16 / 16-byte
// fp32 loads), a wave covers 256 consecutive columns of one row, so every row read is fully coalesced.
#include "dp_common.h"

namespace {

// ------------------------------------------------------------------------------------------------
// element access: VW consecutive elements starting at element index `idx`
// ------------------------------------------------------------------------------------------------
// (non-temporal: every input byte of these kernels is read once and by one workgroup)
typedef uint32_t rw_u32x2 __attribute__((ext_vector_type(2)));
template <bool BF16, int VW>
__device__ __forceinline__ void load_vec(const void* __restrict__ base, size_t idx, float out[VW]) {
    if constexpr (BF16) {
        static_assert(VW == 4, "bf16 rows are read four elements at a time");
        const rw_u32x2 w =
            __builtin_nontemporal_load(reinterpret_cast<const rw_u32x2*>(reinterpret_cast<const uint16_t*>(base) + idx));
        out[0] = dp_bf16_lo(w[0]);
        out[1] = dp_bf16_hi(w[0]);
        out[2] = dp_bf16_lo(w[1]);
        out[3] = dp_bf16_hi(w[1]);
    } else if constexpr (VW == 4) {
        const f32x4_t w = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(reinterpret_cast<const float*>(base) + idx));
        out[0] = w[0]; out[1] = w[1]; out[2] = w[2]; out[3] = w[3];
    } else {
        out[0] = __builtin_nontemporal_load(reinterpret_cast<const float*>(base) + idx);
    }
}

// ------------------------------------------------------------------------------------------------
// column statistics, per example (pass 1)
//   grid (B, ceil(d / (64*VW))), 256 threads = 4 row groups x 64 column lanes
// ------------------------------------------------------------------------------------------------
// Up to COL_MAX_BATCH same-shaped layers per launch (blockIdx.z = layer): the 48 LayerNorms of the model are 3 launches
// per pass instead of 48, and their per-example partials meet in one ordered reduction.
constexpr int COL_MAX_BATCH = 16;
struct ColBatch {
    const void* X[COL_MAX_BATCH];
    const void* G[COL_MAX_BATCH];
};
struct ColOut {
    float* out_x[COL_MAX_BATCH];
    float* out_1[COL_MAX_BATCH];
};
struct ColKeep {
    float* keep[COL_MAX_BATCH];  // per layer: [B][2][d] fp32, the per-example column statistics themselves
};

// out: direct (one layer, one column block): sqnorms, "+="; otherwise partials [B][layers * J], stored.
// KEEP: the statistics of example i (sum_t g x and sum_t g per column: its LayerNorm gain / offset gradient) are also
// written to ck.keep[layer][i], so that pass 2 can weight and add 8 KB per example instead of reading X and G again.
template <bool BF16, int VW, bool USE_X, bool USE_1, bool KEEP>
__global__ __launch_bounds__(256) void colstat_sqnorms_kernel(ColBatch cb, ColKeep ck, int T, int d, float* __restrict__ out,
                                                              int J, int direct) {
    __shared__ float red[4][64][2 * VW];
    __shared__ float wred[4];
    const void* __restrict__ X = cb.X[blockIdx.z];
    const void* __restrict__ G = cb.G[blockIdx.z];
    const int i = blockIdx.x;
    const int lane = threadIdx.x & 63, tg = threadIdx.x >> 6;
    const int col = (blockIdx.y * 64 + lane) * VW;
    float sx[VW], s1[VW];
#pragma unroll
    for (int k = 0; k < VW; ++k) sx[k] = s1[k] = 0.f;
    if (col < d) {
        const size_t base = (size_t)i * T * d + col;
#pragma unroll 4
        for (int t = tg; t < T; t += 4) {
            float g[VW];
            load_vec<BF16, VW>(G, base + (size_t)t * d, g);
            if constexpr (USE_X) {
                float x[VW];
                load_vec<BF16, VW>(X, base + (size_t)t * d, x);
#pragma unroll
                for (int k = 0; k < VW; ++k) sx[k] += g[k] * x[k];
            }
#pragma unroll
            for (int k = 0; k < VW; ++k) s1[k] += g[k];
        }
    }
#pragma unroll
    for (int k = 0; k < VW; ++k) {
        red[tg][lane][k] = sx[k];
        red[tg][lane][VW + k] = s1[k];
    }
    __syncthreads();
    float val = 0.f;
    float sv[2 * VW];
    if (tg == 0) {
#pragma unroll
        for (int k = 0; k < 2 * VW; ++k) {
            sv[k] = (red[0][lane][k] + red[1][lane][k]) + (red[2][lane][k] + red[3][lane][k]);
            const bool on = k < VW ? USE_X : USE_1;
            if (on) val += sv[k] * sv[k];
        }
    }
    const float tot = dp_block_sum<256>(val, wred);
    if (threadIdx.x == 0) {
        if (direct) out[i] += tot;
        else out[((size_t)i * gridDim.z + blockIdx.z) * J + blockIdx.y] = tot;
    }
    // The kept statistics go out last: a store ahead of the reduction's barrier would make every workgroup wait for it.
    if constexpr (KEEP) {
        if (tg == 0 && col < d) {
            float* __restrict__ kp = ck.keep[blockIdx.z] + (size_t)i * 2 * d + col;
            if constexpr (VW == 4) {  // d % 4 == 0 and a 16-byte aligned buffer are checked at the API
                __builtin_nontemporal_store(f32x4_t{sv[0], sv[1], sv[2], sv[3]}, reinterpret_cast<f32x4_t*>(kp));
                __builtin_nontemporal_store(f32x4_t{sv[4], sv[5], sv[6], sv[7]}, reinterpret_cast<f32x4_t*>(kp + d));
            } else {
#pragma unroll
                for (int k = 0; k < VW; ++k) {
                    kp[k] = sv[k];
                    kp[d + k] = sv[VW + k];
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// clip-weighted column sums (pass 2)
//   grid (R, ceil(d / (64*VW))): WG r reduces rows [r*rows_per, (r+1)*rows_per) of the B*T rows
//   partial layout: part[layer][r][0][d] = sum c g x,  part[layer][r][1][d] = sum c g   (blockIdx.z = layer)
// ------------------------------------------------------------------------------------------------
template <bool BF16, int VW, bool USE_X>
// (the clip factors come precomputed: forming them here, a square root and a division per row and thread, cost 2 %)
__global__ __launch_bounds__(256) void colstat_sums_kernel(ColBatch cb, const float* __restrict__ c, int T, int d,
                                                           long nrows, int rows_per, float* __restrict__ part) {
    __shared__ float red[4][64][2 * VW];
    const void* __restrict__ X = cb.X[blockIdx.z];
    const void* __restrict__ G = cb.G[blockIdx.z];
    const int lane = threadIdx.x & 63, tg = threadIdx.x >> 6;
    const int col = (blockIdx.y * 64 + lane) * VW;
    const long r0 = (long)blockIdx.x * rows_per;
    const long r1 = r0 + rows_per < nrows ? r0 + rows_per : nrows;
    float sx[VW], s1[VW];
#pragma unroll
    for (int k = 0; k < VW; ++k) sx[k] = s1[k] = 0.f;
    if (col < d) {
#pragma unroll 4
        for (long r = r0 + tg; r < r1; r += 4) {
            const float w = c[r / T];
            float g[VW];
            load_vec<BF16, VW>(G, (size_t)r * d + col, g);
            if constexpr (USE_X) {
                float x[VW];
                load_vec<BF16, VW>(X, (size_t)r * d + col, x);
#pragma unroll
                for (int k = 0; k < VW; ++k) sx[k] += w * (g[k] * x[k]);
            }
#pragma unroll
            for (int k = 0; k < VW; ++k) s1[k] += w * g[k];
        }
    }
#pragma unroll
    for (int k = 0; k < VW; ++k) {
        red[tg][lane][k] = sx[k];
        red[tg][lane][VW + k] = s1[k];
    }
    __syncthreads();
    if (tg == 0 && col < d) {
        float* p = part + ((size_t)blockIdx.z * gridDim.x + blockIdx.x) * 2 * d;
#pragma unroll
        for (int k = 0; k < VW; ++k) {
            p[col + k] = (red[0][lane][k] + red[1][lane][k]) + (red[2][lane][k] + red[3][lane][k]);
            p[d + col + k] = (red[0][lane][VW + k] + red[1][lane][VW + k]) + (red[2][lane][VW + k] + red[3][lane][VW + k]);
        }
    }
}

// Pass 2 from kept per-example statistics: out_x[j] += sum_i c_i keep[i][0][j], out_1[j] += sum_i c_i keep[i][1][j].
// grid (ceil(2d / 256), layers); 256 threads = 64 float4 columns x 4 example groups; group g adds the examples
// i = g, g+4, ... in ascending order, the four group sums are added as (0+1)+(2+3): fixed order.
__global__ __launch_bounds__(256) void kept_sums_kernel(ColKeep ck, ColOut co, const float* __restrict__ c, int B, int d) {
    __shared__ float4 red[4][64];
    const int lane = threadIdx.x & 63, g = threadIdx.x >> 6;
    const int n4 = 2 * d / 4, d4 = d / 4;
    const int j = blockIdx.x * 64 + lane;
    const float4* __restrict__ src = reinterpret_cast<const float4*>(ck.keep[blockIdx.y]);
    float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
    if (j < n4) {
        int i = g;
        for (; i + 28 < B; i += 32) {
            float4 p[8];
            float w[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                p[u] = src[(size_t)(i + 4 * u) * n4 + j];
                w[u] = c[i + 4 * u];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                t.x += w[u] * p[u].x; t.y += w[u] * p[u].y; t.z += w[u] * p[u].z; t.w += w[u] * p[u].w;
            }
        }
        for (; i < B; i += 4) {
            const float4 p = src[(size_t)i * n4 + j];
            const float w = c[i];
            t.x += w * p.x; t.y += w * p.y; t.z += w * p.z; t.w += w * p.w;
        }
    }
    red[g][lane] = t;
    __syncthreads();
    if (g == 0 && j < n4) {
        const float4 a = red[0][lane], b = red[1][lane], e = red[2][lane], f = red[3][lane];
        float4* dst = j < d4 ? reinterpret_cast<float4*>(co.out_x[blockIdx.y]) + j
                             : reinterpret_cast<float4*>(co.out_1[blockIdx.y]) + (j - d4);
        float4 o = *dst;
        o.x += (a.x + b.x) + (e.x + f.x);
        o.y += (a.y + b.y) + (e.y + f.y);
        o.z += (a.z + b.z) + (e.z + f.z);
        o.w += (a.w + b.w) + (e.w + f.w);
        *dst = o;
    }
}

// out[j] += sum_{r<R} part[r*stride + j], r ascending (fixed order)
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float* __restrict__ part, int R, size_t stride,
                                                              size_t n, float* __restrict__ out) {
    const size_t j = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= n) return;
    float t = 0.f;
    for (int r = 0; r < R; ++r) t += part[(size_t)r * stride + j];
    out[j] += t;
}

__global__ __launch_bounds__(256) void reduce_partials_vec4_kernel(const float4* __restrict__ part, int R,
                                                                   size_t stride4, size_t n4,
                                                                   float4* __restrict__ out) {
    const size_t j = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= n4) return;
    float4 o = out[j];
    float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
    int r = 0;
    // eight independent 16-byte loads in flight per thread; the additions keep the order r = 0, 1, 2, ...
    for (; r + 8 <= R; r += 8) {
        float4 p[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) p[u] = part[(size_t)(r + u) * stride4 + j];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            t.x += p[u].x; t.y += p[u].y; t.z += p[u].z; t.w += p[u].w;
        }
    }
    for (; r < R; ++r) {
        const float4 p = part[(size_t)r * stride4 + j];
        t.x += p.x; t.y += p.y; t.z += p.z; t.w += p.w;
    }
    o.x += t.x; o.y += t.y; o.z += t.z; o.w += t.w;
    out[j] = o;
}

// Few outputs, many partials (column sums): 256 threads = 64 float4 columns x 4 partial groups.  Group g adds
// the partials r = g, g+4, g+8, ... in ascending order; the four group sums are added as (0+1)+(2+3): fixed order.
__global__ __launch_bounds__(256) void reduce_partials_tall_kernel(const float4* __restrict__ part, int R,
                                                                   size_t stride4, size_t n4,
                                                                   float4* __restrict__ out) {
    __shared__ float4 red[4][64];
    const int lane = threadIdx.x & 63, g = threadIdx.x >> 6;
    const size_t j = (size_t)blockIdx.x * 64 + lane;
    float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
    if (j < n4) {
        int r = g;
        for (; r + 28 < R; r += 32) {
            float4 p[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) p[u] = part[(size_t)(r + 4 * u) * stride4 + j];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                t.x += p[u].x; t.y += p[u].y; t.z += p[u].z; t.w += p[u].w;
            }
        }
        for (; r < R; r += 4) {
            const float4 p = part[(size_t)r * stride4 + j];
            t.x += p.x; t.y += p.y; t.z += p.z; t.w += p.w;
        }
    }
    red[g][lane] = t;
    __syncthreads();
    if (g == 0 && j < n4) {
        const float4 a = red[0][lane], b = red[1][lane], c = red[2][lane], d = red[3][lane];
        float4 o = out[j];
        o.x += (a.x + b.x) + (c.x + d.x);
        o.y += (a.y + b.y) + (c.y + d.y);
        o.z += (a.z + b.z) + (c.z + d.z);
        o.w += (a.w + b.w) + (c.w + d.w);
        out[j] = o;
    }
}

// The two column-sum vectors of every layer's partial buffer [R][2][d] in one launch: columns j < d4 go to out_x, the
// others to out_1 (same order of additions as reduce_partials_tall_kernel).
__global__ __launch_bounds__(256) void reduce_partials_pair_kernel(const float4* __restrict__ part, int R, size_t d4,
                                                                   ColOut co) {
    __shared__ float4 red[4][64];
    const int lane = threadIdx.x & 63, g = threadIdx.x >> 6;
    const size_t j = (size_t)blockIdx.x * 64 + lane, n4 = 2 * d4;
    part += (size_t)blockIdx.y * R * n4;  // blockIdx.y = layer
    float4* __restrict__ out_x = reinterpret_cast<float4*>(co.out_x[blockIdx.y]);
    float4* __restrict__ out_1 = reinterpret_cast<float4*>(co.out_1[blockIdx.y]);
    float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
    if (j < n4) {
        int r = g;
        for (; r + 28 < R; r += 32) {
            float4 p[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) p[u] = part[(size_t)(r + 4 * u) * n4 + j];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                t.x += p[u].x; t.y += p[u].y; t.z += p[u].z; t.w += p[u].w;
            }
        }
        for (; r < R; r += 4) {
            const float4 p = part[(size_t)r * n4 + j];
            t.x += p.x; t.y += p.y; t.z += p.z; t.w += p.w;
        }
    }
    red[g][lane] = t;
    __syncthreads();
    if (g == 0 && j < n4) {
        const float4 a = red[0][lane], b = red[1][lane], c = red[2][lane], e = red[3][lane];
        float4* dst = j < d4 ? out_x + j : out_1 + (j - d4);
        float4 o = *dst;
        o.x += (a.x + b.x) + (c.x + e.x);
        o.y += (a.y + b.y) + (c.y + e.y);
        o.z += (a.z + b.z) + (c.z + e.z);
        o.w += (a.w + b.w) + (c.w + e.w);
        *dst = o;
    }
}

// ------------------------------------------------------------------------------------------------
// embedding, per-example norms (pass 1): grid (B, ceil(d/(64*VW))), one wave per workgroup.
// The wave ranks the example's T ids (stable counting rank in LDS), walks the rows in id order and adds
// the square of every run of equal ids, column by column.
// ------------------------------------------------------------------------------------------------
template <bool BF16, int VW, bool DISTINCT>
__global__ __launch_bounds__(64) void embedding_sqnorms_kernel(const int32_t* __restrict__ ids,
                                                               const void* __restrict__ G, int T, int d, int V,
                                                               float* __restrict__ out, int J, int direct,
                                                               int* __restrict__ err) {
    extern __shared__ int32_t lds[];
    int32_t* sid = lds;         // [T] ids of this example
    int32_t* order = lds + T;   // [T] row index at each sorted position
    const int i = blockIdx.x;
    const int lane = threadIdx.x;
    const int col = (blockIdx.y * 64 + lane) * VW;
    bool bad = false;
    for (int t = lane; t < T; t += 64) {
        const int32_t v = ids[(size_t)i * T + t];
        if (v < 0 || v >= V) bad = true;
        sid[t] = v;
    }
    if (bad) atomicOr(err, 1);
    __syncthreads();
    if constexpr (!DISTINCT) {
        for (int t = lane; t < T; t += 64) {
            const int32_t v = sid[t];
            int rank = 0;
            for (int s = 0; s < T; ++s) {
                const int32_t u = sid[s];
                rank += (u < v) || (u == v && s < t);
            }
            order[rank] = t;
        }
        __syncthreads();
    }
    float tot = 0.f;
    if (col < d) {
        const size_t base = (size_t)i * T * d + col;
        if constexpr (DISTINCT) {
#pragma unroll 8
            for (int t = 0; t < T; ++t) {
                float g[VW];
                load_vec<BF16, VW>(G, base + (size_t)t * d, g);
#pragma unroll
                for (int k = 0; k < VW; ++k) tot += g[k] * g[k];
            }
        } else {
            float run[VW];
#pragma unroll
            for (int k = 0; k < VW; ++k) run[k] = 0.f;
            int32_t prev = sid[order[0]];
#pragma unroll 8
            for (int p = 0; p < T; ++p) {
                const int t = order[p];
                const int32_t v = sid[t];
                float g[VW];
                load_vec<BF16, VW>(G, base + (size_t)t * d, g);
                if (v != prev) {
#pragma unroll
                    for (int k = 0; k < VW; ++k) {
                        tot += run[k] * run[k];
                        run[k] = 0.f;
                    }
                    prev = v;
                }
#pragma unroll
                for (int k = 0; k < VW; ++k) run[k] += g[k];
            }
#pragma unroll
            for (int k = 0; k < VW; ++k) tot += run[k] * run[k];
        }
    }
    tot = dp_wave_sum(tot);
    if (lane == 0) {
        // (an out-of-range id only changes the grouping; the error itself is reported by dp_sync)
        if (direct) out[i] += tot;
        else out[(size_t)i * J + blockIdx.y] = tot;
    }
}

// ------------------------------------------------------------------------------------------------
// embedding, clip-weighted scatter (pass 2): stable LSD radix sort of (id, row) + ordered segment sums
// ------------------------------------------------------------------------------------------------
constexpr int SORT_CHUNK = 1024;

__global__ __launch_bounds__(256) void sort_keys_init(const int32_t* __restrict__ ids, int N, int V,
                                                      uint32_t* __restrict__ keys, uint32_t* __restrict__ vals,
                                                      int* __restrict__ err) {
    const int r = blockIdx.x * 256 + threadIdx.x;
    if (r >= N) return;
    const int32_t v = ids[r];
    const bool bad = v < 0 || v >= V;
    if (bad) atomicOr(err, 1);
    keys[r] = bad ? (uint32_t)V : (uint32_t)v;  // sentinel V sorts last and is skipped
    vals[r] = (uint32_t)r;
}

// hist[b * nchunks + c] = number of keys of chunk c whose digit is b (integer counters in LDS: the order of the
// additions does not matter)
__global__ __launch_bounds__(256) void sort_hist(const uint32_t* __restrict__ keys, int N, int shift,
                                                 uint32_t* __restrict__ hist, int nchunks) {
    __shared__ uint32_t cnt[256];
    const int c = blockIdx.x;
    const int n0 = c * SORT_CHUNK;
    const int valid = N - n0 < SORT_CHUNK ? N - n0 : SORT_CHUNK;
    cnt[threadIdx.x] = 0;
    __syncthreads();
    for (int k = threadIdx.x; k < valid; k += 256) atomicAdd(&cnt[(keys[n0 + k] >> shift) & 255u], 1u);
    __syncthreads();
    hist[(size_t)threadIdx.x * nchunks + c] = cnt[threadIdx.x];
}

// In-place exclusive prefix sum of hist[0..n): one workgroup, thread t owns a contiguous slice, read and written as
// 16-byte vectors, eight in flight (n is a multiple of 1024 here: 256 digits x chunks, slices of a multiple of 4).
__global__ __launch_bounds__(256) void sort_scan(uint32_t* __restrict__ hist, int n) {
    __shared__ uint32_t tsum[256];
    const int per = (n + 255) / 256;  // n % 256 == 0: every slice is full
    const int lo = threadIdx.x * per;
    const int hi = lo + per < n ? lo + per : n;
    const bool vec = per % 4 == 0;
    uint32_t s = 0;
    if (vec) {
        const uint4* p4 = reinterpret_cast<const uint4*>(hist + lo);
        const int n4 = (hi - lo) / 4;
        for (int k = 0; k < n4; k += 8) {
            uint4 t[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) t[u] = k + u < n4 ? p4[k + u] : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
            for (int u = 0; u < 8; ++u) s += (t[u].x + t[u].y) + (t[u].z + t[u].w);
        }
    } else {
        for (int k = lo; k < hi; ++k) s += hist[k];
    }
    tsum[threadIdx.x] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t run = 0;
        for (int k = 0; k < 256; ++k) {
            const uint32_t t = tsum[k];
            tsum[k] = run;
            run += t;
        }
    }
    __syncthreads();
    uint32_t run = tsum[threadIdx.x];
    if (vec) {
        uint4* p4 = reinterpret_cast<uint4*>(hist + lo);
        const int n4 = (hi - lo) / 4;
        for (int k = 0; k < n4; k += 8) {
            uint4 t[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) t[u] = k + u < n4 ? p4[k + u] : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                uint4 o;
                o.x = run; run += t[u].x;
                o.y = run; run += t[u].y;
                o.z = run; run += t[u].z;
                o.w = run; run += t[u].w;
                if (k + u < n4) p4[k + u] = o;
            }
        }
    } else {
        for (int k = lo; k < hi; ++k) {
            const uint32_t t = hist[k];
            hist[k] = run;
            run += t;
        }
    }
}

// Stable scatter of one chunk by the current digit.  The chunk is cut into groups of 64 consecutive keys (one wave
// handles a group at a time): digit counts per group (LDS integer counters), an exclusive scan over the groups per
// digit on top of the chunk's global base, and inside a group the rank of a key among the keys of equal digit at lower
// positions, from eight ballots.
__global__ __launch_bounds__(256) void sort_scatter(const uint32_t* __restrict__ keys,
                                                    const uint32_t* __restrict__ vals, int N, int shift,
                                                    const uint32_t* __restrict__ base, int nchunks,
                                                    uint32_t* __restrict__ keys_out, uint32_t* __restrict__ vals_out) {
    constexpr int NG = SORT_CHUNK / 64;  // groups per chunk
    __shared__ uint32_t gcnt[NG][256];
    const int c = blockIdx.x;
    const int n0 = c * SORT_CHUNK;
    const int valid = N - n0 < SORT_CHUNK ? N - n0 : SORT_CHUNK;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int e = threadIdx.x; e < NG * 256; e += 256) (&gcnt[0][0])[e] = 0;
    __syncthreads();
    uint32_t key[NG / 4], val[NG / 4];
#pragma unroll
    for (int q = 0; q < NG / 4; ++q) {
        const int g = wave + 4 * q, k = g * 64 + lane;
        key[q] = val[q] = 0;
        if (k < valid) {
            key[q] = keys[n0 + k];
            val[q] = vals[n0 + k];
            atomicAdd(&gcnt[g][(key[q] >> shift) & 255u], 1u);
        }
    }
    __syncthreads();
    {
        const uint32_t b = threadIdx.x;
        uint32_t run = base[(size_t)b * nchunks + c];
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            const uint32_t t = gcnt[g][b];
            gcnt[g][b] = run;
            run += t;
        }
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < NG / 4; ++q) {
        const int g = wave + 4 * q, k = g * 64 + lane;
        const bool ok = k < valid;
        const uint32_t dgt = (key[q] >> shift) & 255u;
        unsigned long long same = __ballot(ok);
#pragma unroll
        for (int bit = 0; bit < 8; ++bit) {
            const bool one = (dgt >> bit) & 1u;
            const unsigned long long bal = __ballot(ok && one);
            same &= one ? bal : ~bal;
        }
        if (ok) {
            const uint32_t rank = (uint32_t)__popcll(same & ((1ull << lane) - 1ull));
            const uint32_t o = gcnt[g][dgt] + rank;
            keys_out[o] = key[q];
            vals_out[o] = val[q];
        }
    }
}

// Ordered segment sums over the sorted (id, row) list.  Workgroup (pc, cc) = one wave; it owns the
// SEG_CHUNK sorted positions [pc*SEG_CHUNK, ...) and 64*VW columns.  A run of equal ids that lies wholly
// inside the chunk is added to sum_E directly (this workgroup is its only writer).  A run that continues
// from the previous chunk goes to first[pc], a run that starts here and continues into the next chunk goes
// to last[pc]; segment_fixup_kernel adds those pieces in chunk order.
constexpr int SEG_CHUNK = 32;

template <bool BF16, int VW>
__global__ __launch_bounds__(64) void segment_sums_kernel(const uint32_t* __restrict__ keys,
                                                          const uint32_t* __restrict__ vals,
                                                          const void* __restrict__ G, const float* __restrict__ c,
                                                          int N, int T, int d, int V, float* __restrict__ sum_E,
                                                          float* __restrict__ first, float* __restrict__ last) {
    __shared__ uint32_t skey[SEG_CHUNK + 2];  // [0] = key before the chunk, [1..n] = chunk, [n+1] = key after
    __shared__ uint32_t srow[SEG_CHUNK];
    __shared__ float sc[SEG_CHUNK];
    const int pc = blockIdx.x;
    const int lane = threadIdx.x;
    const int p0 = pc * SEG_CHUNK;
    const int n = N - p0 < SEG_CHUNK ? N - p0 : SEG_CHUNK;
    const uint32_t NONE = 0xFFFFFFFFu;
    for (int k = lane; k < n; k += 64) {
        skey[1 + k] = keys[p0 + k];
        const uint32_t row = vals[p0 + k];
        srow[k] = row;
        sc[k] = c[row / (uint32_t)T];
    }
    if (lane == 0) {
        skey[0] = p0 > 0 ? keys[p0 - 1] : NONE;
        skey[n + 1] = p0 + n < N ? keys[p0 + n] : NONE;
    }
    __syncthreads();
    const int col = (blockIdx.y * 64 + lane) * VW;
    if (col >= d) return;
    float acc[VW];
#pragma unroll
    for (int k = 0; k < VW; ++k) acc[k] = 0.f;
    int seg_start = 0;
    for (int k0 = 0; k0 < n; k0 += 8) {
        float g[8][VW];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int k = k0 + u < n ? k0 + u : n - 1;
            load_vec<BF16, VW>(G, (size_t)srow[k] * d + col, g[u]);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int k = k0 + u;
            if (k < n) {
                const uint32_t key = skey[1 + k];
                const float w = sc[k];
#pragma unroll
                for (int e = 0; e < VW; ++e) acc[e] += w * g[u][e];
                if (skey[2 + k] != key) {  // the run ends at position k
                    if (key < (uint32_t)V) {
                        const bool from_prev = seg_start == 0 && skey[0] == key;
                        float* dst = from_prev ? first + (size_t)pc * d + col : sum_E + (size_t)key * d + col;
#pragma unroll
                        for (int e = 0; e < VW; ++e) dst[e] = from_prev ? acc[e] : dst[e] + acc[e];
                    }
#pragma unroll
                    for (int e = 0; e < VW; ++e) acc[e] = 0.f;
                    seg_start = k + 1;
                }
            }
        }
    }
    if (seg_start < n) {
        // the last run continues into the next chunk (skey[n+1] equals its key)
        const uint32_t key = skey[n];
        if (key < (uint32_t)V) {
            const bool from_prev = seg_start == 0 && skey[0] == key;
            float* dst = from_prev ? first + (size_t)pc * d + col : last + (size_t)pc * d + col;
#pragma unroll
            for (int e = 0; e < VW; ++e) dst[e] = acc[e];
        }
    }
}

// Workgroups (pc, column block) for every chunk pc whose last run starts in pc and continues into pc+1: add last[pc],
// then first[q] for the chunks q = pc+1 .. that the run reaches, in that order, and add the total to sum_E[key].
// The end of the run is found by bisection of the sorted keys (the most frequent token spans hundreds of chunks);
// the pieces are then loaded eight at a time and added in chunk order.
__global__ __launch_bounds__(256) void segment_fixup_kernel(const uint32_t* __restrict__ keys, int N, int d, int V,
                                                            int nchunks, const float* __restrict__ first,
                                                            const float* __restrict__ last,
                                                            float* __restrict__ sum_E) {
    const int pc = blockIdx.x;
    const int pend = (pc + 1) * SEG_CHUNK;  // first position of the next chunk
    if (pend >= N) return;
    const uint32_t key = keys[pend - 1];
    if (key >= (uint32_t)V || keys[pend] != key) return;             // no run crosses this boundary
    const int p0 = pc * SEG_CHUNK;
    if (p0 > 0 && keys[p0 - 1] == key && keys[p0] == key) return;    // the run started earlier: not its head
    int lo = pend, hi = N;  // keys[lo] == key; the run ends at the first position in (lo, hi] whose key differs
    while (hi - lo > 1) {
        const int mid = lo + (hi - lo) / 2;
        if (keys[mid] == key) lo = mid;
        else hi = mid;
    }
    const int qlast = lo / SEG_CHUNK;  // every chunk pc+1 .. qlast starts inside the run, so its first[] holds a piece
    const int col = blockIdx.y * 256 + threadIdx.x;
    if (col >= d) return;
    float acc = last[(size_t)pc * d + col];
    int q = pc + 1;
    for (; q + 8 <= qlast + 1; q += 8) {
        float f[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) f[u] = first[(size_t)(q + u) * d + col];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += f[u];
    }
    for (; q <= qlast; ++q) acc += first[(size_t)q * d + col];
    sum_E[(size_t)key * d + col] += acc;
}

inline int bit_length(uint32_t v) {
    int b = 0;
    while (v) {
        ++b;
        v >>= 1;
    }
    return b;
}

inline bool vec4_ok(dp_dtype dt, int d, const void* p, const void* q) {
    if (dt == DP_BF16) return true;  // d % 8 == 0 and 16-byte alignment are checked at the API
    return d % 4 == 0 && (((uintptr_t)p | (uintptr_t)q) & 15) == 0;
}

}  // namespace

// ================================================================================================
// host launchers
// ================================================================================================
dp_status dpk_reduce_partials(dp_ctx* ctx, const float* part, int R, size_t stride, size_t n, float* out) {
    if (n == 0) return DP_OK;
    if (n % 4 == 0 && stride % 4 == 0 && (((uintptr_t)part | (uintptr_t)out) & 15) == 0) {
        const size_t n4 = n / 4;
        if (R >= 32 && n4 <= 16384)
            hipLaunchKernelGGL(reduce_partials_tall_kernel, dim3((unsigned)((n4 + 63) / 64)), dim3(256), 0, ctx->stream,
                               reinterpret_cast<const float4*>(part), R, stride / 4, n4, reinterpret_cast<float4*>(out));
        else
            hipLaunchKernelGGL(reduce_partials_vec4_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0,
                               ctx->stream, reinterpret_cast<const float4*>(part), R, stride / 4, n4,
                               reinterpret_cast<float4*>(out));
    } else {
        hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, ctx->stream, part,
                           R, stride, n, out);
    }
    DP_LAUNCH_CHECK(ctx, "reduce_partials");
    return DP_OK;
}

template <bool BF16, int VW>
static dp_status colstat_sqnorms_launch(dp_ctx* ctx, int L, const void* const* X, const void* const* G, int B, int T, int d,
                                        int use_x, int use_1, float* sqnorms, float* const* keep) {
    const int J = (d + 64 * VW - 1) / (64 * VW);
    ColBatch cb;
    ColKeep ck;
    for (int l = 0; l < COL_MAX_BATCH; ++l) {
        cb.X[l] = use_x ? X[l < L ? l : 0] : nullptr;
        cb.G[l] = G[l < L ? l : 0];
        ck.keep[l] = keep ? keep[l < L ? l : 0] : nullptr;
    }
    float* out = sqnorms;
    int direct = 1;
    if (J > 1 || L > 1) {
        dp_ws_alloc ws(ctx);
        out = ws.get<float>((size_t)B * L * J);
        if (!out) {
            DP_SET_ERR(ctx, "workspace too small for %d x %d norm partials", B, L * J);
            return DP_ERR_WORKSPACE;
        }
        direct = 0;
    }
    dim3 grid(B, J, L);
    if (keep)  // (LayerNorm only: both statistics)
        hipLaunchKernelGGL((colstat_sqnorms_kernel<BF16, VW, true, true, true>), grid, dim3(256), 0, ctx->stream, cb, ck, T, d, out, J, direct);
    else if (use_x && use_1)
        hipLaunchKernelGGL((colstat_sqnorms_kernel<BF16, VW, true, true, false>), grid, dim3(256), 0, ctx->stream, cb, ck, T, d, out, J, direct);
    else if (use_x)
        hipLaunchKernelGGL((colstat_sqnorms_kernel<BF16, VW, true, false, false>), grid, dim3(256), 0, ctx->stream, cb, ck, T, d, out, J, direct);
    else
        hipLaunchKernelGGL((colstat_sqnorms_kernel<BF16, VW, false, true, false>), grid, dim3(256), 0, ctx->stream, cb, ck, T, d, out, J, direct);
    DP_LAUNCH_CHECK(ctx, "colstat_sqnorms");
    if (!direct) return dpk_finish_partials(ctx, out, B, L * J, sqnorms);  // layers, then column blocks, in index order
    return DP_OK;
}

// keep: NULL, or n pointers to [B][2][d] fp32 buffers that receive every example's two statistics (then use_x = use_1 = 1)
dp_status dpk_colstat_sqnorms_batched(dp_ctx* ctx, int n, const void* const* X, const void* const* G, dp_dtype dt, int B, int T,
                                      int d, int use_x, int use_1, float* sqnorms, float* const* keep) {
    if (B == 0 || T == 0 || d == 0 || n == 0 || (!use_x && !use_1)) return DP_OK;
    bool v4 = true;
    for (int l = 0; l < n; ++l) v4 = v4 && vec4_ok(dt, d, use_x ? X[l] : G[l], G[l]);
    for (int l0 = 0; l0 < n; l0 += COL_MAX_BATCH) {
        const int L = n - l0 < COL_MAX_BATCH ? n - l0 : COL_MAX_BATCH;
        const void* const* Xl = use_x ? X + l0 : nullptr;
        dp_status st;
        float* const* kl = keep ? keep + l0 : nullptr;
        if (dt == DP_BF16) st = colstat_sqnorms_launch<true, 4>(ctx, L, Xl, G + l0, B, T, d, use_x, use_1, sqnorms, kl);
        else if (v4) st = colstat_sqnorms_launch<false, 4>(ctx, L, Xl, G + l0, B, T, d, use_x, use_1, sqnorms, kl);
        else st = colstat_sqnorms_launch<false, 1>(ctx, L, Xl, G + l0, B, T, d, use_x, use_1, sqnorms, kl);
        if (st != DP_OK) return st;
    }
    return DP_OK;
}

dp_status dpk_colstat_sqnorms(dp_ctx* ctx, const void* X, const void* G, dp_dtype dt, int B, int T, int d, int use_x,
                              int use_1, float* sqnorms) {
    return dpk_colstat_sqnorms_batched(ctx, 1, &X, &G, dt, B, T, d, use_x, use_1, sqnorms, nullptr);
}

// sum_x[l][j] += sum_i c_i keep[l][i][0][j], sum_1[l][j] += sum_i c_i keep[l][i][1][j]; d % 4 == 0, 16-byte aligned buffers
dp_status dpk_kept_sums_batched(dp_ctx* ctx, int n, float* const* keep, int B, int d, const float* c, float* const* sum_x,
                                float* const* sum_1) {
    if (B == 0 || d == 0 || n == 0) return DP_OK;
    for (int l0 = 0; l0 < n; l0 += COL_MAX_BATCH) {
        const int L = n - l0 < COL_MAX_BATCH ? n - l0 : COL_MAX_BATCH;
        ColKeep ck;
        ColOut co;
        for (int l = 0; l < COL_MAX_BATCH; ++l) {
            ck.keep[l] = keep[l0 + (l < L ? l : 0)];
            co.out_x[l] = sum_x[l0 + (l < L ? l : 0)];
            co.out_1[l] = sum_1[l0 + (l < L ? l : 0)];
        }
        hipLaunchKernelGGL(kept_sums_kernel, dim3((unsigned)((2 * d / 4 + 63) / 64), L), dim3(256), 0, ctx->stream, ck, co, c, B, d);
        DP_LAUNCH_CHECK(ctx, "kept_sums");
    }
    return DP_OK;
}

// out_x / out_1: tables of L pointers, or NULL when that statistic is not wanted (the same for every layer of the call)
template <bool BF16, int VW>
static dp_status colstat_sums_launch(dp_ctx* ctx, int L, const void* const* X, const void* const* G, int B, int T, int d,
                                     const float* c, float* const* out_x, float* const* out_1) {
    const long nrows = (long)B * T;
    const int J = (d + 64 * VW - 1) / (64 * VW);
    long R = 1024 / J;  // about 1024 workgroups per layer
    if (R < 1) R = 1;
    const long maxR = (nrows + 63) / 64;
    if (R > maxR) R = maxR;
    const int rows_per = (int)((nrows + R - 1) / R);
    R = (nrows + rows_per - 1) / rows_per;
    dp_ws_alloc ws(ctx);
    float* part = ws.get<float>((size_t)L * R * 2 * d);
    if (!part) {
        DP_SET_ERR(ctx, "workspace too small for column-sum partials (%d x %ld x 2 x %d floats)", L, R, d);
        return DP_ERR_WORKSPACE;
    }
    ColBatch cb;
    for (int l = 0; l < COL_MAX_BATCH; ++l) {
        cb.X[l] = out_x ? X[l < L ? l : 0] : nullptr;
        cb.G[l] = G[l < L ? l : 0];
    }
    dim3 grid((unsigned)R, J, L);
    if (out_x)
        hipLaunchKernelGGL((colstat_sums_kernel<BF16, VW, true>), grid, dim3(256), 0, ctx->stream, cb, c, T, d, nrows, rows_per, part);
    else
        hipLaunchKernelGGL((colstat_sums_kernel<BF16, VW, false>), grid, dim3(256), 0, ctx->stream, cb, c, T, d, nrows, rows_per, part);
    DP_LAUNCH_CHECK(ctx, "colstat_sums");
    bool pair = out_x && out_1 && d % 4 == 0 && R >= 32 && d <= 32768 && ((uintptr_t)part & 15) == 0;
    for (int l = 0; pair && l < L; ++l) pair = (((uintptr_t)out_x[l] | (uintptr_t)out_1[l]) & 15) == 0;
    if (pair) {
        ColOut co;
        for (int l = 0; l < COL_MAX_BATCH; ++l) {
            co.out_x[l] = out_x[l < L ? l : 0];
            co.out_1[l] = out_1[l < L ? l : 0];
        }
        const size_t d4 = (size_t)d / 4;
        hipLaunchKernelGGL(reduce_partials_pair_kernel, dim3((unsigned)((2 * d4 + 63) / 64), L), dim3(256), 0, ctx->stream,
                           reinterpret_cast<const float4*>(part), (int)R, d4, co);
        DP_LAUNCH_CHECK(ctx, "reduce_partials_pair");
        return DP_OK;
    }
    for (int l = 0; l < L; ++l) {
        const float* pl = part + (size_t)l * R * 2 * d;
        dp_status st = DP_OK;
        if (out_x) st = dpk_reduce_partials(ctx, pl, (int)R, (size_t)2 * d, d, out_x[l]);
        if (st == DP_OK && out_1) st = dpk_reduce_partials(ctx, pl + d, (int)R, (size_t)2 * d, d, out_1[l]);
        if (st != DP_OK) return st;
    }
    return DP_OK;
}

dp_status dpk_colstat_sums_batched(dp_ctx* ctx, int n, const void* const* X, const void* const* G, dp_dtype dt, int B, int T,
                                   int d, const float* c, float* const* out_x, float* const* out_1) {
    if (B == 0 || T == 0 || d == 0 || n == 0 || (!out_x && !out_1)) return DP_OK;
    bool v4 = true;
    for (int l = 0; l < n; ++l) v4 = v4 && vec4_ok(dt, d, out_x ? X[l] : G[l], G[l]);
    for (int l0 = 0; l0 < n; l0 += COL_MAX_BATCH) {
        const int L = n - l0 < COL_MAX_BATCH ? n - l0 : COL_MAX_BATCH;
        const void* const* Xl = out_x ? X + l0 : nullptr;
        float* const* ox = out_x ? out_x + l0 : nullptr;
        float* const* o1 = out_1 ? out_1 + l0 : nullptr;
        dp_status st;
        if (dt == DP_BF16) st = colstat_sums_launch<true, 4>(ctx, L, Xl, G + l0, B, T, d, c, ox, o1);
        else if (v4) st = colstat_sums_launch<false, 4>(ctx, L, Xl, G + l0, B, T, d, c, ox, o1);
        else st = colstat_sums_launch<false, 1>(ctx, L, Xl, G + l0, B, T, d, c, ox, o1);
        if (st != DP_OK) return st;
    }
    return DP_OK;
}

dp_status dpk_colstat_sums(dp_ctx* ctx, const void* X, const void* G, dp_dtype dt, int B, int T, int d, const float* c,
                           float* out_x, float* out_1) {
    return dpk_colstat_sums_batched(ctx, 1, &X, &G, dt, B, T, d, c, out_x ? &out_x : nullptr, out_1 ? &out_1 : nullptr);
}

template <bool BF16, int VW>
static dp_status embedding_sqnorms_launch(dp_ctx* ctx, const int32_t* ids, const void* G, int B, int T, int d, int V,
                                          int distinct, float* sqnorms) {
    const int J = (d + 64 * VW - 1) / (64 * VW);
    float* out = sqnorms;
    int direct = 1;
    if (J > 1) {
        dp_ws_alloc ws(ctx);
        out = ws.get<float>((size_t)B * J);
        if (!out) {
            DP_SET_ERR(ctx, "workspace too small for %d x %d norm partials", B, J);
            return DP_ERR_WORKSPACE;
        }
        direct = 0;
    }
    dim3 grid(B, J);
    const size_t lds = (size_t)2 * T * sizeof(int32_t);
    if (distinct)
        hipLaunchKernelGGL((embedding_sqnorms_kernel<BF16, VW, true>), grid, dim3(64), lds, ctx->stream, ids, G, T, d, V, out, J, direct, ctx->err_word);
    else
        hipLaunchKernelGGL((embedding_sqnorms_kernel<BF16, VW, false>), grid, dim3(64), lds, ctx->stream, ids, G, T, d, V, out, J, direct, ctx->err_word);
    DP_LAUNCH_CHECK(ctx, "embedding_sqnorms");
    if (!direct) return dpk_finish_partials(ctx, out, B, J, sqnorms);
    return DP_OK;
}

dp_status dpk_embedding_sqnorms(dp_ctx* ctx, const int32_t* ids, const void* G, dp_dtype dt, int B, int T, int d, int V,
                                int distinct, float* sqnorms) {
    if (B == 0 || T == 0 || d == 0) return DP_OK;
    if (T > 4096) {
        DP_SET_ERR(ctx, "dp_sqnorms_embedding: T = %d exceeds the supported maximum of 4096", T);
        return DP_ERR_SHAPE;
    }
    if (dt == DP_BF16) return embedding_sqnorms_launch<true, 4>(ctx, ids, G, B, T, d, V, distinct, sqnorms);
    if (vec4_ok(dt, d, G, G)) return embedding_sqnorms_launch<false, 4>(ctx, ids, G, B, T, d, V, distinct, sqnorms);
    return embedding_sqnorms_launch<false, 1>(ctx, ids, G, B, T, d, V, distinct, sqnorms);
}

template <bool BF16, int VW>
static dp_status embedding_sums_launch(dp_ctx* ctx, const int32_t* ids, const void* G, int B, int T, int d, int V,
                                       const float* c, float* sum_E) {
    const long Nl = (long)B * T;
    if (Nl > 0x7FFFFFFFl - SORT_CHUNK) {
        DP_SET_ERR(ctx, "dp_clip_accumulate_embedding: B*T too large");
        return DP_ERR_SHAPE;
    }
    const int N = (int)Nl;
    const int nsort = (N + SORT_CHUNK - 1) / SORT_CHUNK;
    const int nseg = (N + SEG_CHUNK - 1) / SEG_CHUNK;
    dp_ws_alloc ws(ctx);
    uint32_t* k0 = ws.get<uint32_t>(N);
    uint32_t* k1 = ws.get<uint32_t>(N);
    uint32_t* v0 = ws.get<uint32_t>(N);
    uint32_t* v1 = ws.get<uint32_t>(N);
    uint32_t* hist = ws.get<uint32_t>((size_t)256 * nsort);
    float* first = ws.get<float>((size_t)nseg * d);
    float* last = ws.get<float>((size_t)nseg * d);
    if (!k0 || !k1 || !v0 || !v1 || !hist || !first || !last) {
        DP_SET_ERR(ctx, "workspace too small for the embedding sort of %d tokens", N);
        return DP_ERR_WORKSPACE;
    }
    hipLaunchKernelGGL(sort_keys_init, dim3((N + 255) / 256), dim3(256), 0, ctx->stream, ids, N, V, k0, v0, ctx->err_word);
    DP_LAUNCH_CHECK(ctx, "sort_keys_init");
    const int bits = bit_length((uint32_t)V);  // the sentinel V itself must be representable
    for (int shift = 0; shift < bits; shift += 8) {
        hipLaunchKernelGGL(sort_hist, dim3(nsort), dim3(256), 0, ctx->stream, k0, N, shift, hist, nsort);
        hipLaunchKernelGGL(sort_scan, dim3(1), dim3(256), 0, ctx->stream, hist, 256 * nsort);
        hipLaunchKernelGGL(sort_scatter, dim3(nsort), dim3(256), 0, ctx->stream, k0, v0, N, shift, hist, nsort, k1, v1);
        DP_LAUNCH_CHECK(ctx, "radix sort pass");
        uint32_t* t = k0; k0 = k1; k1 = t;
        t = v0; v0 = v1; v1 = t;
    }
    const int J = (d + 64 * VW - 1) / (64 * VW);
    hipLaunchKernelGGL((segment_sums_kernel<BF16, VW>), dim3(nseg, J), dim3(64), 0, ctx->stream, k0, v0, G, c, N, T, d, V, sum_E, first, last);
    DP_LAUNCH_CHECK(ctx, "segment_sums");
    if (nseg > 1) {
        hipLaunchKernelGGL(segment_fixup_kernel, dim3(nseg - 1, (d + 255) / 256), dim3(256), 0, ctx->stream, k0, N, d, V, nseg, first, last, sum_E);
        DP_LAUNCH_CHECK(ctx, "segment_fixup");
    }
    return DP_OK;
}

dp_status dpk_embedding_sums(dp_ctx* ctx, const int32_t* ids, const void* G, dp_dtype dt, int B, int T, int d, int V,
                             const float* c, float* sum_E) {
    if (B == 0 || T == 0 || d == 0) return DP_OK;
    if (dt == DP_BF16) return embedding_sums_launch<true, 4>(ctx, ids, G, B, T, d, V, c, sum_E);
    if (vec4_ok(dt, d, G, G)) return embedding_sums_launch<false, 4>(ctx, ids, G, B, T, d, V, c, sum_E);
    return embedding_sums_launch<false, 1>(ctx, ids, G, B, T, d, V, c, sum_E);
}
