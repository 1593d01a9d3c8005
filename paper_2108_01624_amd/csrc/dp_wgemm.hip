// Clip-weighted dense gradient sum  S_W += sum_i c_i A_i^T G_i = A_flat^T diag(c (x) 1_T) G_flat
// (the sum over the batch of clip(grad, C) in the g_t line of Algorithm 1, for a dense layer whose
// per-example gradient is the outer-product form of Section 4.3), and the tile-by-tile materialisation
// of one example's A_i^T G_i for the squared-norm path that sums squares of the entries.
//
// Both are "TN" contractions: the contraction index (token row k) is the SLOW index of both operands in
// memory, while v_mfma_f32_32x32x16_bf16 wants each lane to hold 8 consecutive k for one output row/column.
// Tiles are staged in LDS as they lie in memory ([k][column], 16-byte chunks) and fragments are fetched
// with the gfx950 transposing LDS read (ds_read_b64_tr_b16): inside a group of 16 lanes, lane i supplies
// the address of 4 adjacent columns of row k0 + i/4 and receives column i of rows k0..k0+3, so two reads
// give a lane its 8 consecutive k.  No permute instructions, natural output layout.
//
// LDS bank conflicts: the four rows a 16-lane group touches are one row pitch (512 B or 256 B) apart, i.e.
// in the same banks.  The 16-byte chunk index is therefore XOR-ed with 4*(row % 4) when a chunk is stored,
// which spreads the four rows of a group, and the two groups of a half-wave, over 256 distinct bytes.
//
// Pipeline per workgroup of the register-staged kernel (8 waves as 2 x 4 on a 256 x 256 tile, or 4 waves as 2 x 2 on
// 128 x 128): global -> registers up to four stages ahead (buffer loads: rows
// past the split's range read as zero, so there is no branch around a load), registers -> LDS ring of
// three stages, LDS -> fragments one 16-row step ahead of the MFMAs, also across the one barrier per stage.
//
// The clip factor c_i multiplies the rows of G in fp32 while they sit in registers between the global load
// and the LDS store (once per element per workgroup); the product is rounded to bf16 (nearest even, by
// v_cvt_pk_bf16_f32); accumulation is fp32 in the MFMA.
//
// Roofline: MFMA.  2*B*T*d_in*d_out flops per layer against (d_in + d_out)*B*T*2 bytes read once.
#include <stdlib.h>

#include <type_traits>

#include "dp_common.h"

namespace {

constexpr int BK = 32;      // token rows per staged tile
constexpr int NSTAGE = 3;   // LDS ring

enum { EPI_STORE = 0, EPI_ADD = 1, EPI_SQNORM = 2 };

struct WgemmArgs {
    const uint16_t* A;   // [K, d_in]
    const uint16_t* G;   // [K, d_out]
    const float* sqnorms;  // [B] squared norms; c_i = min(1, C / sqrt(sqnorms[i])) (unused without scaling)
    float C;
    float* bias_part;    // [nsplit][d_out] column sums of the scaled G rows (written by the tile row 0), or nullptr
    int T, d_in, d_out;
    long K;              // total rows
    long rows_per_split; // multiple of BK (or T for the per-example materialisation)
    int tiles_m, tiles_n, nsplit;
    float* out;          // EPI_STORE: [nsplit][d_in][d_out]; EPI_ADD: [d_in][d_out]; EPI_SQNORM: [nsplit][ntiles]
    int xcd_map;         // 0: plain; 1: split index interleaved over the 8 XCDs; 2: each XCD owns one split and a
                         // rect_m x rect_n-th sub-rectangle of the tile grid; 3 (direct-to-LDS kernel only): the
                         // (unit, tile) sequence cut into 8 equal runs
    int rect_m, rect_n;  // mode 2: the tile grid is cut into rect_m x rect_n rectangles, 8 / nsplit per split;
                         // modes 1 and 3: a unit's tiles are walked in rectangles of this size
    int* err;            // device error word: DP_ERRBIT_NORM is set when a clip factor is NaN (non-finite squared norm)
};

// Several layers of one shape in one launch (direct-to-LDS kernel): the unit of work distribution is the pair
// (layer, row split); `base` describes the common shape, and base.A / base.G / base.out are not used.
constexpr int MAX_BATCH = 32;
struct LayerPtrs {
    const uint16_t* A;
    const uint16_t* G;
    float* out;      // EPI_ADD: the layer's sum_W; EPI_STORE: the layer's first partial [nsplit][d_in][d_out]
    float* sum_b;    // the layer's bias sum buffer or nullptr (device code only tests it; the finish kernel adds)
};
struct WgemmBatchArgs {
    WgemmArgs base;
    int n_layers;
    LayerPtrs L[MAX_BATCH];
};

typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t scale_pair(uint32_t w, float s) {
    const f32x2_t x = {dp_bf16_lo(w) * s, dp_bf16_hi(w) * s};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2_t));  // v_cvt_pk_bf16_f32 (RNE)
}
__device__ __forceinline__ u32x4_t scale_bf16x8(u32x4_t v, float s) {
    u32x4_t o;
    o[0] = scale_pair(v[0], s);
    o[1] = scale_pair(v[1], s);
    o[2] = scale_pair(v[2], s);
    o[3] = scale_pair(v[3], s);
    return o;
}

// 8 consecutive k (rows) of one column, as an MFMA operand: two transposing reads of 4 rows each.
__device__ __forceinline__ bf16x8_t read_frag(const uint16_t* lds_lane_ptr, int row_pitch_elems) {
    typedef s16x4_t __attribute__((address_space(3))) * lptr;
    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lptr)(lds_lane_ptr));
    const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lptr)(lds_lane_ptr + 4 * row_pitch_elems));
    const s16x8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8_t, v);
}

// Workgroup = WVM x WVN waves; wave tile (32*MI) x (32*NI); block tile BM x BN = (32*MI*WVM) x (32*NI*WVN).
// SCALE: multiply G rows by c.  UNIFORM_C: T % BK == 0, so all rows of a stage belong to one example.
template <int MI, int NI, int WVM, int WVN, int EPI, bool SCALE, bool UNIFORM_C>
__global__ __launch_bounds__(64 * WVM * WVN) void wgemm_bf16_kernel(WgemmArgs a) {
    constexpr int NT = 64 * WVM * WVN;
    constexpr int WM = 32 * MI, WN = 32 * NI;
    constexpr int BM = WM * WVM, BN = WN * WVN;
    constexpr int CA = BM / 8, CG = BN / 8;  // 16-byte chunks per tile row
    constexpr int SA = BK * CA / NT, SG = BK * CG / NT;  // staging slots (16-byte chunks) per thread
    static_assert(SA * NT == BK * CA && SG * NT == BK * CG, "tile must divide evenly over the threads");
    __shared__ __attribute__((aligned(16))) uint16_t As[NSTAGE][BK * BM];
    __shared__ __attribute__((aligned(16))) uint16_t Gs[NSTAGE][BK * BN];
    __shared__ float wred[NT / 64];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wr = wave / WVN, wc = wave % WVN;
    const int ntiles = a.tiles_m * a.tiles_n;
    // Workgroup ids are dealt to the 8 XCDs round-robin (id % 8), each XCD with its own L2: give the workgroups
    // of one XCD work that shares operand rows and columns, so that A and G come from HBM about once.
    int tile, split;
    if (a.xcd_map == 1) {
        const int g = blockIdx.x, slot = g >> 3;
        split = (slot / ntiles) * 8 + (g & 7);
        tile = slot % ntiles;
        if (split >= a.nsplit) return;
    } else if (a.xcd_map == 2) {
        const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
        const int nrect = a.rect_m * a.rect_n;
        const int rect = xcd % nrect;
        const int tm = a.tiles_m / a.rect_m, tn = a.tiles_n / a.rect_n;
        split = xcd / nrect;
        tile = ((rect / a.rect_n) * tm + slot / tn) * a.tiles_n + (rect % a.rect_n) * tn + slot % tn;
    } else {
        tile = blockIdx.x % ntiles;
        split = blockIdx.x / ntiles;
    }
    const int pm = tile / a.tiles_n, qn = tile % a.tiles_n;
    const int p0 = pm * BM, q0 = qn * BN;
    const long k_lo = (long)split * a.rows_per_split;
    const long k_hi = k_lo + a.rows_per_split < a.K ? k_lo + a.rows_per_split : a.K;
    const int nrows = k_hi > k_lo ? (int)(k_hi - k_lo) : 0;
    const int nsteps = (nrows + BK - 1) / BK;

    // Buffer resources over this split's rows: any access past the last row returns zero.
    const __amdgpu_buffer_rsrc_t rA = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(a.A + (size_t)k_lo * a.d_in), 0, (int)((size_t)nrows * a.d_in * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t rG = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(a.G + (size_t)k_lo * a.d_out), 0, (int)((size_t)nrows * a.d_out * 2), 0x00020000);

    // Per-thread staging slots: slot j moves the 16-byte chunk at tile row `row`, LDS chunk position `cpos`;
    // the global chunk it holds is cpos ^ swizzle(row).  Columns past the layer width read neighbouring
    // (valid or zero) data and only feed output columns that are never stored.
    int voffA[SA], ldsA[SA], voffG[SG], ldsG[SG], rowG[SG];
#pragma unroll
    for (int j = 0; j < SA; ++j) {
        const int id = tid + NT * j, row = id / CA, cpos = id % CA;
        const int cg = cpos ^ ((row & 3) << 2);
        voffA[j] = (row * a.d_in + p0 + cg * 8) * 2;
        ldsA[j] = row * BM + cpos * 8;
    }
#pragma unroll
    for (int j = 0; j < SG; ++j) {
        const int id = tid + NT * j, row = id / CG, cpos = id % CG;
        const int cg = cpos ^ ((row & 3) << 2);
        voffG[j] = (row * a.d_out + q0 + cg * 8) * 2;
        ldsG[j] = row * BN + cpos * 8;
        rowG[j] = row;
    }
    // Fragment read offsets (elements) inside a stage for k step 0: lane l reads row 8*(l/32) + (l%16)/4
    // (+4 for its second read), columns 32*i + 16*((l/16)%2) + 4*(l%4) .. +3 of operand tile i.
    const int frow = 8 * (lane >> 5) + ((lane & 15) >> 2);
    const int fsw = frow & 3;
    int foffA[MI], foffG[NI];
#pragma unroll
    for (int i = 0; i < MI; ++i) {
        const int col = wr * WM + 32 * i + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
        foffA[i] = frow * BM + (((col >> 3) ^ (fsw << 2)) << 3) + (col & 7);
    }
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int col = wc * WN + 32 * i + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
        foffG[i] = frow * BN + (((col >> 3) ^ (fsw << 2)) << 3) + (col & 7);
    }

    f32x16_t acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    u32x4_t ra[2][SA], rg[2][SG];
    float cs[2][SG];
    // Bias gradient: the workgroups of tile row 0 also sum the scaled G rows they stage, column by column.
    const bool do_bias = SCALE && a.bias_part != nullptr && pm == 0;
    float bsum[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) bsum[e] = 0.f;
    auto gload = [&](int set, int st) {  // stage st -> register set
        const int soffA = st * BK * a.d_in * 2, soffG = st * BK * a.d_out * 2;
#pragma unroll
        for (int j = 0; j < SA; ++j) ra[set][j] = __builtin_amdgcn_raw_buffer_load_b128(rA, voffA[j], soffA, 0);
#pragma unroll
        for (int j = 0; j < SG; ++j) rg[set][j] = __builtin_amdgcn_raw_buffer_load_b128(rG, voffG[j], soffG, 0);
        if constexpr (SCALE) {
            if constexpr (UNIFORM_C) {
                const long k = k_lo + (long)st * BK;
                const float s = dp_clip_factor(a.sqnorms[(uint32_t)(k < a.K ? k : a.K - 1) / (uint32_t)a.T], a.C);
                if (s != s && tid == 0) atomicOr(a.err, DP_ERRBIT_NORM);
#pragma unroll
                for (int j = 0; j < SG; ++j) cs[set][j] = s;
            } else {
#pragma unroll
                for (int j = 0; j < SG; ++j) {
                    long k = k_lo + (long)st * BK + rowG[j];
                    if (k >= a.K) k = a.K - 1;
                    cs[set][j] = dp_clip_factor(a.sqnorms[(uint32_t)k / (uint32_t)a.T], a.C);
                    if (cs[set][j] != cs[set][j]) atomicOr(a.err, DP_ERRBIT_NORM);
                }
            }
        }
    };
    auto lstore = [&](int set, int buf) {
#pragma unroll
        for (int j = 0; j < SA; ++j) *reinterpret_cast<u32x4_t*>(&As[buf][ldsA[j]]) = ra[set][j];
#pragma unroll
        for (int j = 0; j < SG; ++j) {
            u32x4_t v = rg[set][j];
            if constexpr (SCALE) {
                if (do_bias) {
                    // this thread always stages the same 8 columns (see the bias epilogue): add the fp32
                    // products c*g to its running column sums before they are rounded to bf16
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        const float lo = dp_bf16_lo(v[w]) * cs[set][j], hi = dp_bf16_hi(v[w]) * cs[set][j];
                        bsum[2 * w] += lo;
                        bsum[2 * w + 1] += hi;
                        const f32x2_t x = {lo, hi};
                        v[w] = __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2_t));
                    }
                } else {
                    v = scale_bf16x8(v, cs[set][j]);
                }
            }
            *reinterpret_cast<u32x4_t*>(&Gs[buf][ldsG[j]]) = v;
        }
    };
    auto load_frags = [&](int buf, int kk, bf16x8_t* fa, bf16x8_t* fg) {
#pragma unroll
        for (int i = 0; i < MI; ++i) fa[i] = read_frag(&As[buf][kk * 16 * BM + foffA[i]], BM);
#pragma unroll
        for (int i = 0; i < NI; ++i) fg[i] = read_frag(&Gs[buf][kk * 16 * BN + foffG[i]], BN);
    };
    auto mma = [&](const bf16x8_t* fa, const bf16x8_t* fg) {
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fg[j], acc[i][j], 0, 0, 0);
    };

    // The stage count is rounded up to even so that the loop body can be unrolled twice with the register
    // sets fixed at compile time; stages past the range load zeros (buffer bounds) and add nothing.
    const int nsteps2 = (nsteps + 1) & ~1;

    // ---- prologue: stages 0 and 1 into LDS, stages 2 and 3 in flight in registers ----
    bf16x8_t fa0[MI], fg0[NI], fa1[MI], fg1[NI];
    // (the scheduling barriers keep the loads in program order: the compiler's wait counts for the loop
    // are only as tight as the load order on entry is certain)
    gload(0, 0);
    __builtin_amdgcn_sched_barrier(0);
    gload(1, 1);
    __builtin_amdgcn_sched_barrier(0);
    lstore(0, 0);
    gload(0, 2);
    __builtin_amdgcn_sched_barrier(0);
    lstore(1, 1);
    gload(1, 3);
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
    load_frags(0, 0, fa0, fg0);

    // ---- main loop: iteration s computes stage s from LDS[s % 3]; stage s+1 is already visible in
    // LDS[(s+1) % 3]; stage s+2 moves from register set s % 2 into LDS[(s+2) % 3] (the buffer read in
    // iteration s-1, released by that iteration's barrier) and the set is reloaded with stage s+4.
    // There is no branch in the body: everything past the last stage is zeros. ----
    int buf = 0;
    auto body = [&](int s, auto setc) {
        constexpr int SET = decltype(setc)::value;
        const int buf1 = buf == NSTAGE - 1 ? 0 : buf + 1;
        const int buf2 = buf1 == NSTAGE - 1 ? 0 : buf1 + 1;
        load_frags(buf, 1, fa1, fg1);
        mma(fa0, fg0);
        lstore(SET, buf2);
        gload(SET, s + 4);
        load_frags(buf1, 0, fa0, fg0);
        mma(fa1, fg1);
        __syncthreads();
        // nothing of the next iteration may move above this point: its register set is still in flight
        __builtin_amdgcn_sched_barrier(0);
        buf = buf1;
    };
    for (int s = 0; s < nsteps2; s += 2) {
        body(s, std::integral_constant<int, 0>());
        body(s + 1, std::integral_constant<int, 1>());
    }

    if constexpr (SCALE) {
        if (do_bias) {
            // Thread t staged LDS chunk position t % CG of rows t / CG (+ multiples of NT / CG, a multiple of 4),
            // i.e. always the global chunk (t % CG) ^ 4*((t / CG) % 4).  Gather the NT / CG row classes of every
            // column in a fixed order.  The stage buffers are free: the loop ended with a barrier.
            float* scratch = reinterpret_cast<float*>(&As[0][0]);
#pragma unroll
            for (int e = 0; e < 8; ++e) scratch[tid * 8 + e] = bsum[e];
            __syncthreads();
            if (tid < BN && q0 + tid < a.d_out) {
                const int cgl = tid >> 3, e = tid & 7;
                float t = 0.f;
#pragma unroll 4
                for (int r = 0; r < NT / CG; ++r) t += scratch[(r * CG + (cgl ^ ((r & 3) << 2))) * 8 + e];
                a.bias_part[(size_t)split * a.d_out + q0 + tid] = t;
            }
        }
    }

    // MFMA tile (i, j): accumulator register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32.
    if (EPI == EPI_SQNORM) {
        // rows / columns past the layer's widths hold products of neighbouring data: leave them out
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int p = p0 + wr * WM + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
#pragma unroll
                for (int j = 0; j < NI; ++j) {
                    const int q = q0 + wc * WN + 32 * j + (lane & 31);
                    const float v = (p < a.d_in && q < a.d_out) ? acc[i][j][r] : 0.f;
                    s += v * v;
                }
            }
        const float tot = dp_block_sum<NT>(s, wred);
        if (tid == 0) a.out[(size_t)split * ntiles + tile] = tot;
        return;
    }

    float* base = a.out + (EPI == EPI_STORE ? (size_t)split * a.d_in * a.d_out : (size_t)0);
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int p = p0 + wr * WM + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
            if (p < a.d_in) {
#pragma unroll
                for (int j = 0; j < NI; ++j) {
                    const int q = q0 + wc * WN + 32 * j + (lane & 31);
                    if (q < a.d_out) {
                        float* dst = base + (size_t)p * a.d_out + q;
                        if (EPI == EPI_ADD) *dst += acc[i][j][r];
                        else *dst = acc[i][j][r];
                    }
                }
            }
        }
}

// ------------------------------------------------------------------------------------------------
// Fast path of the clip-weighted sum (T a multiple of BK, both widths >= 256): 256 x 256 tile, 8 waves
// (2 x 4, wave tile 128 x 64, accumulators in VGPRs, two waves per SIMD).
//
//  * Both operand tiles go from global memory straight into LDS (buffer_load ... lds, 16 bytes per lane, a wave
//    fills two tile rows per instruction): no staging registers, no LDS store instructions, nothing for the
//    VALU to do per element.  The loads are issued through inline assembly because the compiler would otherwise
//    wait for ALL outstanding LDS-filling loads before every LDS read; here the wave waits (vmcnt) only for the
//    stage it is about to publish and keeps the later stages in flight.  Ring of five 32 KiB stages: all of the CU's LDS.
//  * The clip factor is not applied to the operands at all.  All rows of a stage belong to one example, so the
//    accumulators carry sum_{j<=i} (c_j / c_i) A_j^T G_j: when the stage's example changes they are multiplied
//    by c_prev / c_next (128 + 32 VALU multiplies per wave per example, spread over the two half-iterations
//    around the boundary), and by the last c at the end.  The bf16 products are exact in fp32, so this path is
//    more accurate than rounding c*g to bf16.  Needs whole examples of at least two stages per row split
//    (T a multiple of 64; the host aligns the splits); other shapes take the register-staged kernel.
//  * Bias gradient: column sums of G are one more MFMA with an all-ones A fragment.  Every wave takes that duty
//    for one stage in 2*tiles_m (tile row pm, wave row wr: stages s with s % (2*tiles_m) == 2*pm + wr), so the
//    extra work is spread evenly; the partial sums of (split, pm, wr) are added in a fixed order afterwards.
// ------------------------------------------------------------------------------------------------
constexpr int DMA_NS = 5;  // LDS ring stages (5 x 32 KiB = all 160 KiB of a CU's LDS)

typedef int i32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void dma_load16(i32x4_t rsrc, uint32_t lds_byte_addr, int voff, int soff) {
    // LDS destination of lane l: M0 + 16*l.  voff: per-lane byte offset; soff: wave-uniform byte offset.
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds_byte_addr), "v"(voff), "s"(rsrc), "s"(soff)
                 : "memory", "m0");
}

__device__ __forceinline__ i32x4_t make_rsrc(const void* base, uint32_t bytes) {
    const uint64_t p = (uint64_t)base;
    i32x4_t r;
    r[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)p);
    r[1] = __builtin_amdgcn_readfirstlane((int)(uint32_t)(p >> 32));  // stride 0
    r[2] = __builtin_amdgcn_readfirstlane((int)bytes);
    r[3] = 0x00020000;
    return r;
}

// The kernel uses the 16x16x32 MFMA.  Per flop it moves as many fragment bytes through LDS as 32x32x16 would, but the
// matrix pipe draws less power: a loop of nothing but MFMAs on random operands sustains 2.1 PFLOP/s with this shape
// against 1.4 with 32x32x16 (the chip holds 2.07 against 1.7 GHz; on zeros 2.47 against 1.63 PFLOP/s), and this kernel
// lives under the power limit.  Wave tile 128 x 64 = 8 x 4 tiles of 16 x 16; a stage (32 rows) is one MFMA step per tile,
// worked on in two halves of 16 MFMAs (tile rows 0..3, then 4..7) so that the fragments of the next half arrive while
// this one multiplies: 12 fragments in flight in 48 registers.  Rows r and r + 8 of a stage are read by lanes of the
// same pass, so the chunk swizzle also takes bit 3 of the row.
__device__ __forceinline__ int swz16(int row) { return ((row & 3) << 2) | (((row >> 3) & 1) << 1); }

template <int EPI>
__global__ __launch_bounds__(512) void wgemm_dma16_kernel(WgemmBatchArgs b) {
    constexpr int MI = 8, NI = 4, MH = 4, WVN = 4;  // 16 x 16 tiles per wave: MI x NI, worked on in two halves of MH tile rows
    constexpr int WM = 128, WN = 64, BM = 256, BN = 256;
    constexpr int LPS = 4;  // LDS-filling loads per wave per stage (2 for A, 2 for G)
    __shared__ __attribute__((aligned(16))) uint16_t As[DMA_NS][BK * BM];
    __shared__ __attribute__((aligned(16))) uint16_t Gs[DMA_NS][BK * BN];
    const WgemmArgs& a = b.base;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: everything derived from it stays in SGPRs
    const int wr = wave / WVN, wc = wave % WVN;
    const int ntiles = a.tiles_m * a.tiles_n;
    const int nunits = b.n_layers * a.nsplit;  // unit = layer * nsplit + split
    // Workgroup ids are dealt to the 8 XCDs round-robin: an XCD gets whole units (mode 1) or one rectangle of
    // one unit's tile grid (mode 2), so that its L2 sees each operand row and column about once.
    int tile, unit;
    if (a.xcd_map == 1) {
        // nunits is a multiple of 8: XCD x works through the CONSECUTIVE units x * nunits/8 ... (x+1) * nunits/8 - 1.  With
        // 16-tile units two of them run on an XCD at a time, so neighbouring layers that read the same input (the query
        // and key projections of a block, when the caller hands them one tensor) fetch its panels from HBM once.
        const int g = blockIdx.x, slot = g >> 3;
        unit = (g & 7) * (nunits >> 3) + slot / ntiles;
        if (unit >= nunits) return;
        // An XCD runs about 32 workgroups at a time: walk the unit's tile grid in rect_m x rect_n rectangles so
        // that those 32 share as many operand columns as possible (rect 1 x 1 = plain row-major order).
        const int t = slot % ntiles, per = a.rect_m * a.rect_n, rect = t / per, w = t % per;
        const int rpr = a.tiles_n / a.rect_n;
        tile = ((rect / rpr) * a.rect_m + w / a.rect_n) * a.tiles_n + (rect % rpr) * a.rect_n + w % a.rect_n;
    } else if (a.xcd_map == 2) {
        const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
        const int nrect = a.rect_m * a.rect_n;
        const int rect = xcd % nrect;
        const int tm = a.tiles_m / a.rect_m, tn = a.tiles_n / a.rect_n;
        unit = xcd / nrect;
        tile = ((rect / a.rect_n) * tm + slot / tn) * a.tiles_n + (rect % a.rect_n) * tn + slot % tn;
    } else {
        // mode 3: the (unit, tile) pairs in unit-major order, cut into 8 equal runs, one per XCD: balanced for any
        // unit and tile count; at most 7 units have their tiles on two XCDs
        const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
        const int total = nunits * ntiles, per_xcd = (total + 7) >> 3;
        const int w = xcd * per_xcd + slot;
        if (slot >= per_xcd || w >= total) return;
        unit = w / ntiles;
        const int t = w - unit * ntiles, per = a.rect_m * a.rect_n, rect = t / per, r = t % per;
        const int rpr = a.tiles_n / a.rect_n;
        tile = ((rect / rpr) * a.rect_m + r / a.rect_n) * a.tiles_n + (rect % rpr) * a.rect_n + r % a.rect_n;
    }
    const int layer = unit / a.nsplit, split = unit % a.nsplit;
    const uint16_t* Aptr = b.L[layer].A;
    const uint16_t* Gptr = b.L[layer].G;
    const int pm = tile / a.tiles_n, qn = tile % a.tiles_n;
    const int p0 = pm * BM, q0 = qn * BN;
    const long k_lo = (long)split * a.rows_per_split;
    const long k_hi = k_lo + a.rows_per_split < a.K ? k_lo + a.rows_per_split : a.K;
    const int nrows = k_hi > k_lo ? (int)(k_hi - k_lo) : 0;
    const int nsteps = (nrows + BK - 1) / BK;

    const i32x4_t rA = make_rsrc(Aptr + (size_t)k_lo * a.d_in, (uint32_t)((size_t)nrows * a.d_in * 2));
    const i32x4_t rG = make_rsrc(Gptr + (size_t)k_lo * a.d_out, (uint32_t)((size_t)nrows * a.d_out * 2));

    // Load j (0, 1) of this wave fills tile rows 4*wave + 2*j and + 1: lane l -> row + l/32, LDS chunk l%32,
    // which holds global chunk (l%32) ^ swz16(row).
    int voffA[2], voffG[2];
    uint32_t ldsA[2], ldsG[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int row0 = 4 * wave + 2 * j, row = row0 + (lane >> 5);
        const int cg = (lane & 31) ^ swz16(row);
        voffA[j] = (row * a.d_in + p0 + cg * 8) * 2;
        voffG[j] = (row * a.d_out + q0 + cg * 8) * 2;
        ldsA[j] = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint16_t*)&As[0][row0 * BM];
        ldsG[j] = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint16_t*)&Gs[0][row0 * BN];
    }
    auto issue = [&](int st, int buf) {
        // stages past the range load the last stage again (never multiplied): the stage offset is not part of the
        // buffer bounds check, so it must not run past the rows
        const int stc = st < nsteps ? st : (nsteps > 0 ? nsteps - 1 : 0);
        const int soffA = __builtin_amdgcn_readfirstlane(stc * BK * a.d_in * 2);
        const int soffG = __builtin_amdgcn_readfirstlane(stc * BK * a.d_out * 2);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            dma_load16(rA, __builtin_amdgcn_readfirstlane(ldsA[j] + buf * (BK * BM * 2)), voffA[j], soffA);
            dma_load16(rG, __builtin_amdgcn_readfirstlane(ldsG[j] + buf * (BK * BN * 2)), voffG[j], soffG);
        }
    };
    // Operand of the 16x16x32 MFMA: lane l holds the 8 consecutive k = 8*(l/16) .. +7 of column l%16 of its tile.  The
    // transposing read hands lane i of a 16-lane group column i of the 4 rows x 16 columns that the group addresses
    // (lane i: row i/4, columns 4*(i%4) .. +3): two reads, rows frow and frow + 4 (same swizzle: bits 0, 1, 3 agree).
    const int frow = 8 * (lane >> 4) + ((lane & 15) >> 2);
    const int fsw = swz16(frow);
    int foffA[MI], foffG[NI];
#pragma unroll
    for (int i = 0; i < MI; ++i) {
        const int col = wr * WM + 16 * i + 4 * (lane & 3);
        foffA[i] = frow * BM + (((col >> 3) ^ fsw) << 3) + (col & 7);
    }
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int col = wc * WN + 16 * i + 4 * (lane & 3);
        foffG[i] = frow * BN + (((col >> 3) ^ fsw) << 3) + (col & 7);
    }
    auto load_fa = [&](int buf, int half, bf16x8_t* fa) {
#pragma unroll
        for (int i = 0; i < MH; ++i) fa[i] = read_frag(&As[buf][foffA[half * MH + i]], BM);
    };

    f32x4_t acc[MI][NI], bacc[NI];
#pragma unroll
    for (int j = 0; j < NI; ++j) {
#pragma unroll
        for (int r = 0; r < 4; ++r) bacc[j][r] = 0.f;
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.f;
    }
    const bool want_bias = b.L[layer].sum_b != nullptr;
    const int duty_mod = 2 * a.tiles_m, duty = 2 * pm + wr;
    const uint32_t one2 = 0x3F803F80u;  // two bf16 ones
    const bf16x8_t ones = __builtin_bit_cast(bf16x8_t, u32x4_t{one2, one2, one2, one2});
    auto mma_bias = [&](const bf16x8_t* fg) {
#pragma unroll
        for (int j = 0; j < NI; ++j) bacc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, fg[j], bacc[j], 0, 0, 0);
    };
    // fragments of one stage: tile rows 0..3 (lo), 4..7 (hi) of A and the four tile columns of G
    bf16x8_t fa_lo[MH], fa_hi[MH], fg[NI];
    float c_cur = 1.f;  // clip factor of the example being accumulated (set by the example's first stage)

    // prologue: DMA_NS - 1 stages in flight; publish stage 0
    constexpr int AHEAD = DMA_NS - 1;  // the newest stage in flight is AHEAD stages past the one being multiplied
#pragma unroll
    for (int st = 0; st < AHEAD; ++st) issue(st, st);
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((AHEAD - 1) * LPS) : "memory");  // stage 0 has landed
    __syncthreads();
    int buf = 0;      // ring slot of the stage being multiplied
    int ibuf = AHEAD; // ring slot the next load fills
    load_fa(buf, 0, fa_lo);
#pragma unroll
    for (int j = 0; j < NI; ++j) fg[j] = read_frag(&Gs[buf][foffG[j]], BN);

    // One loop iteration = one stage = one barrier.
    int duty_ctr = 0;  // (index of the stage being multiplied) % duty_mod
    const int spe = a.T / BK;                                  // stages per example (>= 2)
    int ex_run = (int)((uint32_t)k_lo / (uint32_t)a.T);        // the next example to start (row splits begin on examples)
    const int nex = (int)(a.K / a.T);
    // lane l: clip factor c_e of example e = (ex & ~63) + l and the rescaling ratio c_{e-1} / c_e that applies when
    // example e starts.  Two plain loads per 64 examples; the compiler's wait for them also waits for the
    // LDS-filling loads in flight, a bubble once per 256 or more stages.
    float cvec = 1.f, rvec = 1.f;
    auto load_factors = [&](int ex) {
        const int e = (ex & ~63) + lane;
        const float n_e = e < nex ? a.sqnorms[e] : 1.f;
        const float n_p = (e >= 1 && e - 1 < nex) ? a.sqnorms[e - 1] : n_e;
        cvec = dp_clip_factor(n_e, a.C);
        rvec = dp_clip_factor(n_p, a.C) / cvec;
        if (cvec != cvec) atomicOr(a.err, DP_ERRBIT_NORM);  // NaN factor: this unit's sums become NaN as well
    };
    if (nsteps > 0) load_factors(ex_run);
    int s_issue = AHEAD;
    // Rescaling at an example boundary (every accumulator register times c_prev / c_next) is spread over the two halves
    // around it: in the second half of the example's last stage (PRE) a tile of the first half is multiplied in every
    // MFMA slot and a tile of the second half two MFMAs after its own MFMA; the last two tiles directly before their
    // MFMAs in the second half of the next example's first stage (POST).  Every stage kind is a straight-line body.
    constexpr int PLAIN = 0, POST = 1, PRE = 2;
    float ratio = 1.f;  // c_prev / c_next of the boundary being worked on (set in PRE, used up in POST)
    auto scale_tile = [&](int i, int j) {
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[i][j][r] *= ratio;
    };
    auto body = [&](auto kind_tag) {
        constexpr int KIND = decltype(kind_tag)::value;
        const int buf1 = buf + 1 == DMA_NS ? 0 : buf + 1;
        const bool bias_now = want_bias && duty_ctr == duty;
        duty_ctr = duty_ctr + 1 == duty_mod ? 0 : duty_ctr + 1;
        load_fa(buf, 1, fa_hi);  // needed by the second half
        if (KIND == POST) {
            // first stage of example ex_run: take over the example's factor
            const int el = __builtin_amdgcn_readfirstlane(ex_run & 63);
            c_cur = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, cvec), el));
            ++ex_run;
        }
        // first half: tile rows 0..3, tile column by tile column
#pragma unroll
        for (int t = 0; t < MH * NI; ++t) {
            const int i = t % MH, j = t / MH;
            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa_lo[i], fg[j], acc[i][j], 0, 0, 0);
        }
        if (KIND == POST) {
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) bacc[j][r] *= ratio;
        }
        if (bias_now) mma_bias(fg);
        __builtin_amdgcn_s_setprio(0);
        // my loads of the next stage have landed (later stages may still be in flight); after the barrier every
        // wave's have, and every wave has finished reading the stage whose ring slot the newest stage now overwrites
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((AHEAD - 2) * LPS) : "memory");
        __syncthreads();
        load_fa(buf1, 0, fa_lo);  // the next stage's first half
        if (KIND == PRE) {
            // last stage of example ex_run - 1; the factors of 64 examples sit in registers (lane = example mod 64)
            if ((ex_run & 63) == 0) load_factors(ex_run);
            const int el = __builtin_amdgcn_readfirstlane(ex_run & 63);
            ratio = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, rvec), el));
        }
        // second half: tile rows 4..7.  When a tile column is done its G fragment makes room for the next stage's,
        // and one of the four LDS-filling loads of the newest stage goes out (spread, not back to back: issued
        // together by all eight waves they queue up in the address unit).
        {
            // of the two waves that share a SIMD, the one in the half that also issues the fills goes first (+3 %
            // measured; raising the priority in the first half as well costs 1 %)
            __builtin_amdgcn_s_setprio(1);
            const int stc = s_issue < nsteps ? s_issue : (nsteps > 0 ? nsteps - 1 : 0);
            const int soffA = __builtin_amdgcn_readfirstlane(stc * BK * a.d_in * 2);
            const int soffG = __builtin_amdgcn_readfirstlane(stc * BK * a.d_out * 2);
#pragma unroll
            for (int t = 0; t < MH * NI; ++t) {
                const int i = MH + t % MH, j = t / MH;
                if (KIND == POST && t >= MH * NI - 2) {
                    __builtin_amdgcn_sched_barrier(0);
                    scale_tile(i, j);
                    __builtin_amdgcn_sched_barrier(0);
                }
                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa_hi[t % MH], fg[j], acc[i][j], 0, 0, 0);
                if (t % MH == MH - 1) {
                    const int jj = j >> 1;
                    __builtin_amdgcn_sched_barrier(0);
                    fg[j] = read_frag(&Gs[buf1][foffG[j]], BN);
                    if ((j & 1) == 0)
                        dma_load16(rA, __builtin_amdgcn_readfirstlane(ldsA[jj] + ibuf * (BK * BM * 2)), voffA[jj], soffA);
                    else
                        dma_load16(rG, __builtin_amdgcn_readfirstlane(ldsG[jj] + ibuf * (BK * BN * 2)), voffG[jj], soffG);
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (KIND == PRE) {
                    __builtin_amdgcn_sched_barrier(0);
                    scale_tile(t % MH, t / MH);
                    if (t >= 2) scale_tile(MH + (t - 2) % MH, (t - 2) / MH);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        __builtin_amdgcn_s_setprio(0);
        ++s_issue;
        ibuf = ibuf + 1 == DMA_NS ? 0 : ibuf + 1;
        buf = buf1;
    };
    // The unit's rows are whole examples (the host aligns row splits to examples), at least two stages each.
    const int n_ex_unit = nsteps / spe;
    for (int e = 0; e + 1 < n_ex_unit; ++e) {
        body(std::integral_constant<int, POST>{});
        for (int q = 0; q < spe - 2; ++q) body(std::integral_constant<int, PLAIN>{});
        body(std::integral_constant<int, PRE>{});
    }
    if (n_ex_unit > 0) {
        body(std::integral_constant<int, POST>{});
        for (int q = 0; q < spe - 1; ++q) body(std::integral_constant<int, PLAIN>{});
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // nothing may still be writing LDS when the workgroup ends

    // MFMA tile (i, j): accumulator register r of lane l holds row 4*(l/16) + r, column l%16.
    float* base = b.L[layer].out + (EPI == EPI_STORE ? (size_t)split * a.d_in * a.d_out : (size_t)0);
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int p = p0 + wr * WM + 16 * i + 4 * (lane >> 4) + r;
            if (p < a.d_in) {
#pragma unroll
                for (int j = 0; j < NI; ++j) {
                    const int q = q0 + wc * WN + 16 * j + (lane & 15);
                    if (q < a.d_out) {
                        float* dst = base + (size_t)p * a.d_out + q;
                        if (EPI == EPI_ADD) *dst += acc[i][j][r] * c_cur;
                        else *dst = acc[i][j][r] * c_cur;
                    }
                }
            }
        }
    if (want_bias && lane < 16) {
        // every row of the ones-product equals the column sums; row 0 sits in register 0 of lanes 0..15
        float* bp = a.bias_part + ((size_t)(unit * a.tiles_m + pm) * 2 + wr) * a.d_out;
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const int q = q0 + wc * WN + 16 * j + lane;
            if (q < a.d_out) bp[q] = bacc[j][0] * c_cur;
        }
    }
}

// Calibration: the clip-weighted GEMM's matrix work with nothing around it - 32 accumulator tiles of 16 x 16 per wave
// (128 registers), 8 + 4 operand fragments that stay in registers, 32 MFMAs per iteration, 8 waves per workgroup (two
// per SIMD), one workgroup per CU.  Operands are pseudo-random bf16 values in +-[1, 2) (the rate the chip sustains
// depends on the data: on zeros it holds a higher clock).  What this loop sustains is the ceiling of any kernel that
// executes these MFMAs on this card under its power limit.
__global__ __launch_bounds__(512) void mfma_ceiling_kernel(int iters, float* __restrict__ sink) {
    constexpr int MI = 8, NI = 4;
    const uint32_t t = blockIdx.x * 512u + threadIdx.x;
    auto rnd = [&](uint32_t k) {  // two bf16 values with random sign and mantissa, exponent 0
        uint32_t h = (t * 0x9E3779B1u) ^ (k * 0x85EBCA77u);
        h ^= h >> 15; h *= 0x2C1B3C6Du; h ^= h >> 12; h *= 0x297A2D39u; h ^= h >> 15;
        return (h & 0x807F807Fu) | 0x3F803F80u;
    };
    bf16x8_t fa[MI], fg[NI];
#pragma unroll
    for (int i = 0; i < MI; ++i) fa[i] = __builtin_bit_cast(bf16x8_t, u32x4_t{rnd(8 * i), rnd(8 * i + 1), rnd(8 * i + 2), rnd(8 * i + 3)});
#pragma unroll
    for (int j = 0; j < NI; ++j) fg[j] = __builtin_bit_cast(bf16x8_t, u32x4_t{rnd(100 + 8 * j), rnd(101 + 8 * j), rnd(102 + 8 * j), rnd(103 + 8 * j)});
    f32x4_t acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[i], fg[j], acc[i][j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j) s += (acc[i][j][0] + acc[i][j][1]) + (acc[i][j][2] + acc[i][j][3]);
    sink[t] = s;
}

// sum_b[layer][q] += sum over the layer's nb partial rows, in row order (fixed order).  grid (n_layers, d_out/256).
__global__ __launch_bounds__(256) void bias_finish_kernel(WgemmBatchArgs b, int nb) {
    const int layer = blockIdx.x;
    float* dst = b.L[layer].sum_b;
    const int q = blockIdx.y * 256 + threadIdx.x;
    if (!dst || q >= b.base.d_out) return;
    const float* src = b.base.bias_part + (size_t)layer * nb * b.base.d_out + q;
    float t = 0.f;
    for (int r = 0; r < nb; ++r) t += src[(size_t)r * b.base.d_out];
    dst[q] += t;
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

template <int MI, int NI, int WVM, int WVN, int EPI, bool SCALE, bool UNIFORM_C>
void wgemm_launch(dp_ctx* ctx, const WgemmArgs& a, unsigned grid) {
    hipLaunchKernelGGL((wgemm_bf16_kernel<MI, NI, WVM, WVN, EPI, SCALE, UNIFORM_C>), dim3(grid),
                       dim3(64 * WVM * WVN), 0, ctx->stream, a);
}

// Tile configurations: 0 = 128 x 128 (4 waves of 64 x 64), 2 = 256 x 256 with 8 waves of 128 x 64 (two waves per
// SIMD, which lets one wave's MFMAs run under the other's loads, conversions and waits).
template <int EPI, bool SCALE>
void wgemm_dispatch(dp_ctx* ctx, const WgemmArgs& a, unsigned grid, int cfg, bool uniform) {
    if (cfg == 2) {
        if (uniform) wgemm_launch<4, 2, 2, 4, EPI, SCALE, true>(ctx, a, grid);
        else wgemm_launch<4, 2, 2, 4, EPI, SCALE, false>(ctx, a, grid);
    } else {
        if (uniform) wgemm_launch<2, 2, 2, 2, EPI, SCALE, true>(ctx, a, grid);
        else wgemm_launch<2, 2, 2, 2, EPI, SCALE, false>(ctx, a, grid);
    }
}

}  // namespace

// Tile shape: 256 x 256 when both dimensions are at least that large, otherwise 128 x 128.
static inline bool big_tile(int d_in, int d_out) { return d_in >= 256 && d_out >= 256; }
// The direct-to-LDS kernel serves the 256 x 256 tile when all rows of a stage share one example.
static inline bool use_dma_path(int cfg, bool uniform) { return cfg != 0 && uniform; }
static inline int tile_cfg(int d_in, int d_out) { return big_tile(d_in, d_out) ? 2 : 0; }

// A split's rows of one operand must stay below 2^31 bytes (32-bit buffer offsets).
static inline bool range_ok(long rows, int d_in, int d_out) {
    const long w = d_in > d_out ? d_in : d_out;
    return (rows + 4 * BK) * w * 2 < (1l << 31);
}

namespace {
// The row splits' partial sums of all layers of a launch, added in one launch: blockIdx.y = layer,
// out_l[j] += sum_{r<R} part_l[r*n4 + j] with r ascending (a fixed order).
struct ReduceBatch {
    const float4* part[MAX_BATCH];
    float4* out[MAX_BATCH];
};
__global__ __launch_bounds__(256) void reduce_layers_kernel(ReduceBatch rb, int R, size_t n4) {
    const size_t j = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= n4) return;
    const float4* __restrict__ part = rb.part[blockIdx.y];
    float4* __restrict__ out = rb.out[blockIdx.y];
    float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
    int r = 0;
    for (; r + 4 <= R; r += 4) {  // four independent 16-byte loads in flight; additions stay in order
        float4 p[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) p[u] = part[(size_t)(r + u) * n4 + j];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            t.x += p[u].x; t.y += p[u].y; t.z += p[u].z; t.w += p[u].w;
        }
    }
    for (; r < R; ++r) {
        const float4 p = part[(size_t)r * n4 + j];
        t.x += p.x; t.y += p.y; t.z += p.z; t.w += p.w;
    }
    float4 o = out[j];
    o.x += t.x; o.y += t.y; o.z += t.z; o.w += t.w;
    out[j] = o;
}
}  // namespace

// Row-split count of one launch of the direct-to-LDS kernel over `nl` layers of `ntiles` tiles: the count with the
// smallest modelled time.  An XCD runs 32 workgroups at a time and gets an eighth of the launch's workgroups, so
// the launch takes ceil(workgroups / 8 / 32) rounds of one workgroup's time (1 us per step of BK rows at the rate
// the kernel sustains, plus 8 us of prologue and epilogue); more than one split sends partial sums through memory
// (written once, read once, about 4 TB/s) and costs one reduction launch.  `spe`: stages per example
// (splits start on examples).
static long choose_nsplit_dma(int nl, int ntiles, long ksteps, long spe, int d_in, int d_out) {
    const long max_split = ksteps / 8 < 1 ? 1 : ksteps / 8;
    long best = 1;
    double best_t = 0.0;
    for (long s = 1; s <= max_split && s <= 64; ++s) {
        const long steps_per = ((ksteps + s - 1) / s + spe - 1) / spe * spe;
        const long se = (ksteps + steps_per - 1) / steps_per;  // the splits that are not empty
        if (se != s && s > 1) continue;                        // the same plan as a smaller s
        const long per_xcd = ((long)nl * se * ntiles + 7) / 8;
        const long rounds = (per_xcd + 31) / 32;
        double t = (double)rounds * ((double)steps_per + 8.0);
        if (se > 1) t += (double)nl * (double)(se + 2) * d_in * d_out * 4.0 / 4.0e6 + 6.0;
        if (s == 1 || t < best_t) {
            best = se;
            best_t = t;
        }
    }
    return best;
}

// Clip-weighted sums of n same-shaped dense layers.  Layers that the direct-to-LDS kernel can take (bf16, both
// widths >= 256, T a multiple of the stage height) go out in launches of up to MAX_BATCH layers; anything else
// falls back to one call per layer.
dp_status dpk_weighted_gemm_batched(dp_ctx* ctx, int n, const void* const* A, const void* const* G, dp_dtype dt, int B,
                                    int T, int d_in, int d_out, const float* sqnorms, float C, float* const* sum_W,
                                    float* const* sum_b) {
    const bool dma = dt == DP_BF16 && d_in > 0 && use_dma_path(tile_cfg(d_in, d_out), T % (2 * BK) == 0);
    if (!dma) {
        for (int l = 0; l < n; ++l) {
            dp_status st = dpk_weighted_gemm(ctx, A[l], G[l], dt, B, T, d_in, d_out, sqnorms, C, sum_W[l], sum_b ? sum_b[l] : nullptr);
            if (st != DP_OK) return st;
        }
        return DP_OK;
    }
    const long K = (long)B * T;
    const long ksteps = (K + BK - 1) / BK;
    // layers per launch: enough to give every CU one workgroup, but no more than one round of workgroups when a
    // layer has many tiles (workgroups that run at the same time share operands through L2; later rounds do not)
    const int tiles_per_layer = ((d_in + 255) / 256) * ((d_out + 255) / 256);
    int per_launch = 256 / tiles_per_layer;
    if (per_launch < 1) per_launch = 1;
    if (per_launch > MAX_BATCH) per_launch = MAX_BATCH;
    for (int l0 = 0; l0 < n; l0 += per_launch) {
        const int nl = n - l0 < per_launch ? n - l0 : per_launch;
        WgemmBatchArgs b;
        WgemmArgs& a = b.base;
        a.A = nullptr;
        a.G = nullptr;
        a.out = nullptr;
        a.sqnorms = sqnorms;
        a.C = C;
        a.err = ctx->err_word;
        a.T = T;
        a.d_in = d_in;
        a.d_out = d_out;
        a.K = K;
        a.tiles_m = (d_in + 255) / 256;
        a.tiles_n = (d_out + 255) / 256;
        const int ntiles = a.tiles_m * a.tiles_n;
        const long spe = T / BK;  // row splits begin on examples: the kernel rescales across example boundaries only
        long nsplit = choose_nsplit_dma(nl, ntiles, ksteps, spe, d_in, d_out);
        while (!range_ok((ksteps + nsplit - 1) / nsplit * BK, d_in, d_out)) nsplit *= 2;
        bool any_bias = false;
        for (int l = 0; l < nl; ++l)
            if (sum_b && sum_b[l0 + l]) any_bias = true;
        // partial sums [nl][nsplit][d_in][d_out] and bias partials (one row per unit, tile row and wave row):
        // fewer splits until the workspace holds both
        dp_ws_alloc ws(ctx);
        float* part = nullptr;
        float* bias_part = nullptr;
        for (;;) {
            ws.off = ctx->ws_base;
            part = nsplit > 1 ? ws.get<float>((size_t)nl * nsplit * d_in * d_out) : nullptr;
            bias_part = any_bias ? ws.get<float>((size_t)nl * nsplit * a.tiles_m * 2 * d_out) : nullptr;
            if ((nsplit == 1 || part) && (!any_bias || bias_part)) break;
            if (nsplit == 1) {
                DP_SET_ERR(ctx, "workspace too small for the bias partials");
                return DP_ERR_WORKSPACE;
            }
            nsplit = nsplit > 8 ? nsplit - 8 : nsplit / 2;
        }
        const long steps_per = ((ksteps + nsplit - 1) / nsplit + spe - 1) / spe * spe;
        a.rows_per_split = steps_per * BK;
        if (!range_ok(a.rows_per_split, d_in, d_out)) {
            DP_SET_ERR(ctx, "dp_clip_accumulate_dense: workspace too small to split %ld rows", K);
            return DP_ERR_WORKSPACE;
        }
        nsplit = (ksteps + steps_per - 1) / steps_per;
        a.nsplit = (int)nsplit;
        const long nunits = (long)nl * nsplit;
        // whole units dealt to the XCDs when that is balanced; otherwise equal runs of the (unit, tile) sequence
        a.xcd_map = nunits % 8 == 0 ? 1 : 3;
        a.rect_m = a.rect_n = 1;
        if (nunits < 8 && 8 % nunits == 0) {
            // 8 / nunits rectangles per unit: the cut with the smallest half-perimeter (operand bytes per XCD)
            const int nrect = 8 / (int)nunits;
            int best = -1;
            for (int rm = 1; rm <= nrect; ++rm) {
                if (nrect % rm) continue;
                const int rn = nrect / rm;
                if (a.tiles_m % rm || a.tiles_n % rn) continue;
                const int cost = a.tiles_m / rm + a.tiles_n / rn;
                if (best < 0 || cost < best) {
                    best = cost;
                    a.rect_m = rm;
                    a.rect_n = rn;
                }
            }
            if (best >= 0) a.xcd_map = 2;
        }
        if (a.xcd_map != 2 && ntiles > 32) {
            // rectangle of about 32 tiles (one XCD's worth of workgroups) with the smallest half-perimeter
            int best = -1;
            for (int tm = 1; tm <= a.tiles_m && tm <= 32; ++tm) {
                if (a.tiles_m % tm) continue;
                int tn = 32 / tm;
                if (tn > a.tiles_n) tn = a.tiles_n;
                while (tn > 1 && a.tiles_n % tn) --tn;
                const int cost = (tm + tn) * 1024 / (tm * tn);  // operand columns fetched per tile
                if (best < 0 || cost < best) {
                    best = cost;
                    a.rect_m = tm;
                    a.rect_n = tn;
                }
            }
        }
        const long nwg = a.xcd_map == 3 ? (nunits * ntiles + 7) / 8 * 8 : nunits * ntiles;
        if (nwg > 0x7FFFFFFFl) {
            DP_SET_ERR(ctx, "dp_clip_accumulate_dense: too many tiles");
            return DP_ERR_SHAPE;
        }
        b.n_layers = nl;
        for (int l = 0; l < MAX_BATCH; ++l) {
            const int src = l0 + (l < nl ? l : 0);
            b.L[l].A = (const uint16_t*)A[src];
            b.L[l].G = (const uint16_t*)G[src];
            b.L[l].out = nsplit == 1 ? sum_W[src] : part + (size_t)l * nsplit * d_in * d_out;
            b.L[l].sum_b = sum_b ? sum_b[src] : nullptr;
        }
        const int nb = (int)nsplit * a.tiles_m * 2;  // bias partial rows per layer
        a.bias_part = bias_part;
        {
            dp_prof_scope prof(ctx, DP_PROF_WGEMM, 2.0 * (double)K * d_in * d_out * nl);
            const dim3 grid((unsigned)nwg), block(512);
            if (nsplit == 1) hipLaunchKernelGGL((wgemm_dma16_kernel<EPI_ADD>), grid, block, 0, ctx->stream, b);
            else hipLaunchKernelGGL((wgemm_dma16_kernel<EPI_STORE>), grid, block, 0, ctx->stream, b);
        }
        DP_LAUNCH_CHECK(ctx, "wgemm_dma");
        if (nsplit > 1) {
            ReduceBatch rb;
            for (int l = 0; l < MAX_BATCH; ++l) {
                rb.part[l] = reinterpret_cast<const float4*>(b.L[l < nl ? l : 0].out);
                rb.out[l] = reinterpret_cast<float4*>(sum_W[l0 + (l < nl ? l : 0)]);
            }
            const size_t n4 = (size_t)d_in * d_out / 4;  // d_out is a multiple of 8
            hipLaunchKernelGGL(reduce_layers_kernel, dim3((unsigned)((n4 + 255) / 256), nl), dim3(256), 0, ctx->stream,
                               rb, (int)nsplit, n4);
            DP_LAUNCH_CHECK(ctx, "reduce_layers");
        }
        if (any_bias) {
            hipLaunchKernelGGL(bias_finish_kernel, dim3(nl, (d_out + 255) / 256), dim3(256), 0, ctx->stream, b, nb);
            DP_LAUNCH_CHECK(ctx, "bias_finish");
        }
    }
    return DP_OK;
}

dp_status dpk_mfma_ceiling(dp_ctx* ctx, int iters, int launches, double* tflops) {
    int cus = 0;
    DP_HIP_CHECK(ctx, hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, ctx->device));
    if (cus <= 0) cus = 256;
    dp_ws_alloc ws(ctx);
    float* sink = ws.get<float>((size_t)cus * 512);
    if (!sink) {
        DP_SET_ERR(ctx, "workspace too small for the calibration kernel");
        return DP_ERR_WORKSPACE;
    }
    hipEvent_t e0, e1;
    DP_HIP_CHECK(ctx, hipEventCreate(&e0));
    if (hipEventCreate(&e1) != hipSuccess) {
        (void)hipEventDestroy(e0);
        DP_SET_ERR(ctx, "hipEventCreate failed");
        return DP_ERR_HIP;
    }
    hipLaunchKernelGGL(mfma_ceiling_kernel, dim3(cus), dim3(512), 0, ctx->stream, iters, sink);  // warm-up
    hipError_t e = hipEventRecord(e0, ctx->stream);
    for (int l = 0; l < launches; ++l) hipLaunchKernelGGL(mfma_ceiling_kernel, dim3(cus), dim3(512), 0, ctx->stream, iters, sink);
    if (e == hipSuccess) e = hipGetLastError();
    if (e == hipSuccess) e = hipEventRecord(e1, ctx->stream);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e != hipSuccess) {
        DP_SET_ERR(ctx, "mfma calibration failed: %s", hipGetErrorString(e));
        return DP_ERR_HIP;
    }
    const double flops = (double)launches * cus * 8.0 * (double)iters * 32.0 * (2.0 * 16 * 16 * 32);
    *tflops = ms > 0.f ? flops / (ms * 1e-3) / 1e12 : 0.0;
    return DP_OK;
}

dp_status dpk_weighted_gemm(dp_ctx* ctx, const void* A, const void* G, dp_dtype dt, int B, int T, int d_in, int d_out,
                            const float* sqnorms, float C, float* sum_W, float* sum_b) {
    const long K = (long)B * T;
    if (dt == DP_F32) {
        dp_status st = dpk_clip_factors(ctx, sqnorms, B, C, ctx->cbuf);
        if (st != DP_OK) return st;
        if (d_in > 0) {
            dim3 grid((d_out + 63) / 64, (d_in + 63) / 64);
            hipLaunchKernelGGL(wgemm_f32_kernel, grid, dim3(256), 0, ctx->stream, (const float*)A, (const float*)G,
                               ctx->cbuf, T, K, d_in, d_out, sum_W);
            DP_LAUNCH_CHECK(ctx, "wgemm_f32");
        }
        if (sum_b) return dpk_colstat_sums(ctx, nullptr, G, dt, B, T, d_out, ctx->cbuf, nullptr, sum_b);
        return DP_OK;
    }
    if (d_in == 0) {  // no weights: only the bias sums are left
        if (!sum_b) return DP_OK;
        dp_status st = dpk_clip_factors(ctx, sqnorms, B, C, ctx->cbuf);
        if (st != DP_OK) return st;
        return dpk_colstat_sums(ctx, nullptr, G, dt, B, T, d_out, ctx->cbuf, nullptr, sum_b);
    }
    if (use_dma_path(tile_cfg(d_in, d_out), T % (2 * BK) == 0))
        return dpk_weighted_gemm_batched(ctx, 1, &A, &G, dt, B, T, d_in, d_out, sqnorms, C, &sum_W, &sum_b);
    const bool big = big_tile(d_in, d_out);
    const int BM = big ? 256 : 128, BN = BM;
    WgemmArgs a;
    a.A = (const uint16_t*)A;
    a.G = (const uint16_t*)G;
    a.sqnorms = sqnorms;
    a.C = C;
    a.err = ctx->err_word;
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
        else if (nsplit > 4) nsplit = max_split >= 8 ? 8 : 4;
        else if (nsplit == 3) nsplit = 4;
        if (nsplit > max_split) nsplit = max_split < 1 ? 1 : max_split;
        if (nsplit < 1) nsplit = 1;
    }
    while (!range_ok((ksteps + nsplit - 1) / nsplit * BK, d_in, d_out)) nsplit *= 2;
    // partial sums [nsplit][d_in][d_out] and bias partials [nsplit][d_out]: fewer splits until the workspace holds both
    dp_ws_alloc ws(ctx);
    float* part = nullptr;
    float* bias_part = nullptr;
    for (;;) {
        ws.off = ctx->ws_base;
        part = nsplit > 1 ? ws.get<float>((size_t)nsplit * d_in * d_out) : nullptr;
        bias_part = sum_b ? ws.get<float>((size_t)nsplit * d_out) : nullptr;
        if ((nsplit == 1 || part) && (!sum_b || bias_part)) break;
        if (nsplit == 1) {
            DP_SET_ERR(ctx, "workspace too small for the bias partials");
            return DP_ERR_WORKSPACE;
        }
        nsplit = nsplit > 8 ? nsplit - 8 : nsplit / 2;
    }
    const long steps_per = (ksteps + nsplit - 1) / nsplit;
    a.rows_per_split = steps_per * BK;
    if (!range_ok(a.rows_per_split, d_in, d_out)) {
        DP_SET_ERR(ctx, "dp_clip_accumulate_dense: workspace too small to split %ld rows", K);
        return DP_ERR_WORKSPACE;
    }
    nsplit = (ksteps + steps_per - 1) / steps_per;
    a.nsplit = (int)nsplit;
    a.xcd_map = nsplit >= 8 ? 1 : 0;
    a.rect_m = a.rect_n = 1;
    if (nsplit < 8 && 8 % nsplit == 0) {
        // 8 / nsplit rectangles per split: pick the cut with the smallest half-perimeter (operand bytes per XCD)
        const int nrect = 8 / (int)nsplit;
        int best = -1;
        for (int rm = 1; rm <= nrect; ++rm) {
            if (nrect % rm) continue;
            const int rn = nrect / rm;
            if (a.tiles_m % rm || a.tiles_n % rn) continue;
            const int cost = a.tiles_m / rm + a.tiles_n / rn;
            if (best < 0 || cost < best) {
                best = cost;
                a.rect_m = rm;
                a.rect_n = rn;
            }
        }
        if (best >= 0) a.xcd_map = 2;
    }
    a.bias_part = bias_part;
    const long nwg = a.xcd_map == 1 ? ((nsplit + 7) / 8) * 8 * ntiles : nsplit * ntiles;
    if (nwg > 0x7FFFFFFFl) {
        DP_SET_ERR(ctx, "dp_clip_accumulate_dense: too many tiles");
        return DP_ERR_SHAPE;
    }
    const bool uniform = T % BK == 0;
    const double flops = 2.0 * (double)K * d_in * d_out;
    const int cfg = tile_cfg(d_in, d_out);
    if (nsplit == 1) {
        a.out = sum_W;
        dp_prof_scope prof(ctx, DP_PROF_WGEMM, flops);
        wgemm_dispatch<EPI_ADD, true>(ctx, a, (unsigned)nwg, cfg, uniform);
    } else {
        a.out = part;
        dp_prof_scope prof(ctx, DP_PROF_WGEMM, flops);
        wgemm_dispatch<EPI_STORE, true>(ctx, a, (unsigned)nwg, cfg, uniform);
    }
    DP_LAUNCH_CHECK(ctx, "wgemm_bf16");
    dp_status st = DP_OK;
    if (nsplit > 1)
        st = dpk_reduce_partials(ctx, part, (int)nsplit, (size_t)d_in * d_out, (size_t)d_in * d_out, sum_W);
    if (st == DP_OK && sum_b) st = dpk_reduce_partials(ctx, a.bias_part, (int)nsplit, (size_t)d_out, (size_t)d_out, sum_b);
    return st;
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
        a.sqnorms = nullptr;
        a.C = 1.f;
        a.err = ctx->err_word;
        a.bias_part = nullptr;
        a.T = T;
        a.d_in = d_in;
        a.d_out = d_out;
        a.K = (long)B * T;
        a.tiles_m = (d_in + BM - 1) / BM;
        a.tiles_n = (d_out + BN - 1) / BN;
        a.nsplit = B;  // one "split" per example: rows [i*T, (i+1)*T)
        a.rows_per_split = T;
        a.xcd_map = 0;
        a.rect_m = a.rect_n = 1;
        if (!range_ok(T, d_in, d_out)) {
            DP_SET_ERR(ctx, "dp_sqnorms_dense: one example's activations exceed 2 GiB");
            return DP_ERR_SHAPE;
        }
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
        wgemm_dispatch<EPI_SQNORM, false>(ctx, a, (unsigned)nwg, tile_cfg(d_in, d_out), true);
        DP_LAUNCH_CHECK(ctx, "wgemm_bf16 (materialise)");
        st = dpk_finish_partials(ctx, part, B, ntiles, sqnorms);
    }
    if (st != DP_OK) return st;
    if (has_bias) return dpk_colstat_sqnorms(ctx, nullptr, G, dt, B, T, d_out, 0, 1, sqnorms);
    return DP_OK;
}
