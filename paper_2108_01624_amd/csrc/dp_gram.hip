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
#include <stdlib.h>

#include <type_traits>

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

// ------------------------------------------------------------------------------------------------
// T <= 128 (one block per example), both widths multiples of 64: the same computation with the row panels
// streamed straight into a four-stage LDS ring by LDS-filling buffer loads, three 16 KiB chunks in flight per
// workgroup (the register-staged kernel above keeps one: at two workgroups per CU that is too few bytes in
// flight to cover the HBM latency at full bandwidth).  The loads go through inline assembly so that the wave
// waits (vmcnt) for the chunk it is about to publish only, not for every load in flight.
// LDS layout: [128 rows][8 chunks of 16 B], chunk position c of row r holds global chunk c ^ ((r >> 1) & 7):
// the 16-byte reads of 16 consecutive rows then fall into 64 distinct banks.
// ------------------------------------------------------------------------------------------------
typedef int gram_i32x4 __attribute__((ext_vector_type(4)));

// STREAM: non-temporal hint, for data that no other workgroup reads again (every byte of a T <= 128 example is read
// once; +4 % there).  The units of a longer example share their panels through L2 and must not use it.
template <bool STREAM>
__device__ __forceinline__ void gram_dma16(gram_i32x4 rsrc, uint32_t lds_byte_addr, int voff, int soff) {
    if (STREAM)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen nt lds"
                     :
                     : "s"(lds_byte_addr), "v"(voff), "s"(rsrc), "s"(soff)
                     : "memory", "m0");
    else
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                     :
                     : "s"(lds_byte_addr), "v"(voff), "s"(rsrc), "s"(soff)
                     : "memory", "m0");
}

__device__ __forceinline__ gram_i32x4 gram_rsrc(const void* base, uint32_t bytes) {
    const uint64_t p = (uint64_t)base;
    gram_i32x4 r;
    r[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)p);
    r[1] = __builtin_amdgcn_readfirstlane((int)(uint32_t)(p >> 32));
    r[2] = __builtin_amdgcn_readfirstlane((int)bytes);
    r[3] = 0x00020000;
    return r;
}

// GDK: contraction chunk per stage (a row segment of 2*GDK bytes per load); NS: ring stages.
// Up to GRAM_MAX_BATCH same-shaped layers per launch: workgroup g works on example g % B of layer g / B.  More
// workgroups than the chip holds at once keep the memory pipeline full across examples (one round of 512
// workgroups spends a fifth of its time filling and draining it).
constexpr int GRAM_MAX_BATCH = 16;
struct GramBatch {
    const uint16_t* A[GRAM_MAX_BATCH];
    const uint16_t* G[GRAM_MAX_BATCH];
    // layers that share their input (Q, K, V of one block): entry l stands for n_out layers with input A[l] and
    // output gradients G[l], G2[l], G3[l].  Their norms add up to <A A^T (+1), sum_j G_j G_j^T>, so A A^T is formed
    // once and the G_j chunks all go into one accumulator (T <= 128 kernel only).
    const uint16_t* G2[GRAM_MAX_BATCH];
    const uint16_t* G3[GRAM_MAX_BATCH];
    int n_out;
    int n_layers;
    int B;
};

// out: n_layers == 1: sqnorms, "+="; otherwise partials [B][n_layers], stored.
template <int GDK, int NS, int WGS_PER_CU>
__global__ __launch_bounds__(256, WGS_PER_CU) void gram_dma_kernel(GramBatch gb, int T, int d_in, int d_out,
                                                                   int has_bias, float* __restrict__ out) {
    constexpr int STAGE = GB * GDK;        // bf16 elements per stage
    constexpr int CPR = GDK / 8;           // 16-byte chunks per row (8 or 16)
    constexpr int RPI = 64 / CPR;          // rows filled by one wave-wide load
    constexpr int LPS = GB / RPI / 4;      // loads per wave per stage
    __shared__ __attribute__((aligned(16))) uint16_t ring[NS][STAGE];
    __shared__ float wred[4];
    const int layer = blockIdx.x / gb.B, i = blockIdx.x - layer * gb.B;
    const uint16_t* __restrict__ A = gb.A[layer];
    const uint16_t* __restrict__ G = gb.G[layer];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave >> 1, wc = wave & 1;
    const bool active = wr <= wc;  // the lower-left quadrant mirrors the upper-right one
    const bool diagw = wr == wc;   // ... and inside a diagonal quadrant the lower-left 32 x 32 tile the upper-right one
    const int nchA = d_in / GDK, nchG1 = d_out / GDK, nch = nchA + gb.n_out * nchG1;
    // chunk position c of row r holds global chunk c ^ swz(r): 16 consecutive rows -> 64 distinct banks
    auto swz = [](int r) { return CPR == 8 ? (r >> 1) & 7 : r & 15; };

    // rows >= T of the panel lie outside the example's byte range and read as zero
    const gram_i32x4 rA = gram_rsrc(A + (size_t)i * T * d_in, (uint32_t)((size_t)T * d_in * 2));
    const gram_i32x4 rG = gram_rsrc(G + (size_t)i * T * d_out, (uint32_t)((size_t)T * d_out * 2));
    const gram_i32x4 rG2 = gram_rsrc((gb.n_out > 1 ? gb.G2[layer] : G) + (size_t)i * T * d_out, (uint32_t)((size_t)T * d_out * 2));
    const gram_i32x4 rG3 = gram_rsrc((gb.n_out > 2 ? gb.G3[layer] : G) + (size_t)i * T * d_out, (uint32_t)((size_t)T * d_out * 2));
    // load j of this wave fills rows (LPS*wave + j)*RPI .. : lane l -> row + l/CPR, chunk position l%CPR
    int voffA[LPS], voffG[LPS];
    uint32_t ldsoff[LPS];
#pragma unroll
    for (int j = 0; j < LPS; ++j) {
        const int row0 = (LPS * wave + j) * RPI, row = row0 + lane / CPR;
        const int cg = (lane % CPR) ^ swz(row);
        voffA[j] = (row * d_in + cg * 8) * 2;
        voffG[j] = (row * d_out + cg * 8) * 2;
        ldsoff[j] = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint16_t*)&ring[0][row0 * GDK];
    }
    int ibuf = 0;  // buffer of the next stage to issue
    const int rotA = i % nchA, rotG = i % nchG1;
    auto issue = [&](int st) {
        const bool isA = st < nchA;
        const int cgi = st - nchA;                                             // chunk index over all output gradients
        const int which = cgi >= 2 * nchG1 ? 2 : (cgi >= nchG1 ? 1 : 0);       // which of the (up to three) tensors
        // The chunks of a tensor are taken in an order rotated by the example index: the contraction does not care, and
        // workgroups that start together (and advance in step) then read different column ranges at any moment.  With one
        // order for all, every workgroup reads the same 256 bytes of rows that lie 2-8 KiB apart, i.e. the same few memory
        // channels (+12 % bandwidth on 1024 x 4096 layers, +2 % on 1024 x 1024).
        const int c0 = isA ? st : cgi - which * nchG1, nc = isA ? nchA : nchG1, r0 = isA ? rotA : rotG;
        const int cr = c0 + r0 >= nc ? c0 + r0 - nc : c0 + r0;
        const int soff = __builtin_amdgcn_readfirstlane(cr * GDK * 2);
        // one choice of the source per stage, then a straight run of loads (every descriptor is a variable of its own
        // and stays in scalar registers; with the choice inside the loop each load of an output-gradient stage went
        // through a chain of branches)
        auto run = [&](const gram_i32x4& rs, const int (&voff)[LPS], int so) {
#pragma unroll
            for (int j = 0; j < LPS; ++j)
                gram_dma16<true>(rs, __builtin_amdgcn_readfirstlane(ldsoff[j] + ibuf * (STAGE * 2)), voff[j], so);
        };
        if (isA) run(rA, voffA, soff);
        else if (st >= nch) run(rG, voffG, 0x7FFFFFF0);  // past the end: reads zeros, keeps the load count uniform
        else if (which == 0) run(rG, voffG, soff);
        else if (which == 1) run(rG2, voffG, soff);
        else run(rG3, voffG, soff);
        ibuf = ibuf + 1 == NS ? 0 : ibuf + 1;
    };
    // fragment addresses (elements) inside a stage for k step 0
    int fr[2], fc[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int r = wr * 64 + u * 32 + (lane & 31), c = wc * 64 + u * 32 + (lane & 31);
        fr[u] = r * GDK + (((lane >> 5) ^ swz(r)) << 3);
        fc[u] = c * GDK + (((lane >> 5) ^ swz(c)) << 3);
    }
    f32x16_t accA[2][2], accG[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) accA[a][b][r] = accG[a][b][r] = 0.f;

#pragma unroll
    for (int st = 0; st < NS - 1; ++st) issue(st);
    int cbuf = 0, s = 0;
    // The multiply of one stage is straight-line code: which Gram matrix it feeds and whether the wave owns a diagonal
    // quadrant are decided outside it (a branch per MFMA pair otherwise).
    auto compute = [&](f32x16_t (&acc)[2][2], auto diag_tag) {
        constexpr bool DG = decltype(diag_tag)::value;
        const uint16_t* st = ring[cbuf];
#pragma unroll
        for (int kk = 0; kk < GDK / 16; ++kk) {
            bf16x8_t a0[2], b0[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                // k chunk 2*kk + lane/32: its swizzled position differs from the kk = 0 one by XOR 2*kk
                const int xr = fr[u] ^ ((2 * kk) << 3), xc = fc[u] ^ ((2 * kk) << 3);
                a0[u] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(st + xr));
                b0[u] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(st + xc));
            }
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int nt = 0; nt < 2; ++nt)
                    if (!(DG && mt == 1 && nt == 0))
                        acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0[mt], b0[nt], acc[mt][nt], 0, 0, 0);
        }
    };
    auto phase = [&](int end, f32x16_t (&acc)[2][2]) {
        for (; s < end; ++s) {
            // my loads of chunk s have landed (later chunks may be in flight); after the barrier everyone's have,
            // and everyone is done reading chunk s-1, whose buffer the newest chunk overwrites
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 2) * LPS) : "memory");
            __syncthreads();
            issue(s + NS - 1);
            if (active) {
                if (diagw) compute(acc, std::true_type{});
                else compute(acc, std::false_type{});
            }
            cbuf = cbuf + 1 == NS ? 0 : cbuf + 1;
        }
    };
    phase(nchA, accA);
    phase(nch, accG);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // nothing may still be writing LDS when the workgroup ends
    const float bias_term = has_bias ? 1.f : 0.f;
    float sum = 0.f;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                sum += (a == 0 && b == 1 && diagw ? 2.f : 1.f) * ((accA[a][b][r] + bias_term) * accG[a][b][r]);  // skipped tiles hold zeros
    sum *= wr == wc ? 1.f : (wr < wc ? 2.f : 0.f);
    const float tot = dp_block_sum<256>(sum, wred);
    if (threadIdx.x == 0) {
        if (gb.n_layers == 1) out[i] += tot;
        else out[(size_t)i * gb.n_layers + layer] = tot;
    }
}

// ------------------------------------------------------------------------------------------------
// T > 128, widths multiples of 64: the panels of a 64-wide contraction chunk go straight into an LDS ring (no staging
// registers, no LDS store instructions), as in the kernel above.  At this size the contraction, not HBM, is the bound on
// paper (T flop per byte against ~310 at the machine balance); in practice it is the path that fills the LDS (a CU takes
// about 120 GB/s from L2 this way, and a panel costs 16 KiB per stage) together with the matrix pipe.  A
// workgroup of 8 waves (two per SIMD, one workgroup per CU) works on a UNIT of cells of the example's T x T plane, cut into
// 128 x 128 cells of which only the upper triangle is formed (by symmetry a cell (R, C) with C < R stands for (C, R)):
//  * a DIAGONAL BLOCK: the three cells (a, a), (a, b), (b, b) of two neighbouring panels a, b = a + 1 - two panel fills
//    for three cells.  The two diagonal cells need only the tiles on and above their diagonals, so the block has 136
//    tiles of 16 x 16 where two full cells have 128, and they fit the same registers: cut into 64-wide strips the block
//    is a 4 x 4 triangle of quadrants; waves 0-5 take the six quadrants off the diagonal (16 tiles each), waves 6 and 7
//    two diagonal quadrants each (2 x 10 tiles; both operands of such a quadrant are the same fragments).
//  * a ROW PAIR: two cells (R, C1), (R, C2) that share their row panel R, which is filled once for both: three panel fills
//    where two workgroups with a cell each fill four (two when the leading cell is the diagonal one, C1 == R).  Waves 0-3
//    own the 64 x 64 quadrants of the first cell, waves 4-7 those of the second; a leading diagonal cell skips its
//    lower-left quadrant and the mirrored tiles of its diagonal quadrants.
// Over the upper triangle of a 4 x 4 plane that is 2 blocks and 2 row pairs: 10 panel fills and 4 workgroups where a
// workgroup per cell needs 16 and 10.  A ring that uses all of the LDS for stages in flight (three stages of 48 KiB
// for three panels, five of 32 KiB for two) covers the latency of the fills: every panel comes from HBM once, the units
// of an example share it through L2.
// ------------------------------------------------------------------------------------------------
constexpr int GU_K = 64;         // contraction chunk per stage
constexpr int GU_LDS = 5 * 2 * GB * GU_K;  // bf16 elements of the ring: 160 KiB, all of a CU's LDS
// Ring stages by the number of panels a stage holds (48, 32 or 16 KiB a stage): a fill that misses L2 takes a few
// microseconds, so a unit with fewer panels per stage runs further ahead.
__host__ __device__ constexpr int gu_stages(int npl) { return npl == 3 ? 3 : (npl == 2 ? 5 : 10); }
constexpr int GU_MAX_BLK = 16;   // T <= 2048
constexpr int GU_MAX_UNITS = GU_MAX_BLK * (GU_MAX_BLK + 1) / 4 + 1;
struct GramUnits {
    int n_units;
    // row pair: R | C1 << 8 | C2 << 16 (C2 == 255: the unit has one cell only); diagonal block of panels a, b: a | a << 8 | b << 16 | 1 << 24
    uint32_t rc[GU_MAX_UNITS];
};

// NPL: panels filled per stage (1: a diagonal cell alone; 2: a diagonal block, a diagonal cell + one more of its row, or
// one off-diagonal cell; 3: two off-diagonal cells).  BLK: the unit is a diagonal block (cells (R, R), (R, C2), (C2, C2)).
template <int NPL, bool BLK>
__device__ __forceinline__ float gram_unit_ring(const uint16_t* __restrict__ A, const uint16_t* __restrict__ G, int T, int d_in,
                                                int d_out, int R, int C1, int C2, float bias_term, uint16_t* ring) {
    static_assert(!BLK || NPL == 2, "a diagonal block has two panels");
    constexpr int PANEL = GB * GU_K;   // bf16 elements of one panel of a stage
    constexpr int STAGE = NPL * PANEL; // ... of one stage: its NPL panels side by side
    constexpr int GU_NS = gu_stages(NPL);
    static_assert(GU_NS * STAGE <= GU_LDS, "ring exceeds the LDS array");
    constexpr int LPP = 2;             // loads per wave per panel: 8 rows of 8 chunks each, 16 loads a panel
    constexpr int LPS = NPL * LPP;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cell = wave >> 2, wr = (wave >> 1) & 1, wc = wave & 1;
    const bool diag0 = C1 == R, two = C2 != 255;
    // panels of a stage, in this order: rows R; rows C1 when the first cell is off the diagonal; rows C2 when there is a second cell
    const bool active = BLK || (cell == 0 ? (!diag0 || wr <= wc) : two);
    const bool diagw = !BLK && cell == 0 && diag0 && wr == wc;  // a diagonal quadrant of a diagonal cell: tiles below its diagonal mirror those above
    const bool twodiag = BLK && wave >= 6;                      // two diagonal quadrants of a diagonal block
    const int nchA = d_in / GU_K, nch = nchA + d_out / GU_K;
    auto swz = [](int r) { return (r >> 1) & 7; };
    // rows >= T lie outside the example's byte range and read as zero
    const gram_i32x4 rA = gram_rsrc(A, (uint32_t)((size_t)T * d_in * 2));
    const gram_i32x4 rG = gram_rsrc(G, (uint32_t)((size_t)T * d_out * 2));
    // load j of this wave fills rows (LPP*wave + j)*8 .. +7 of a panel: lane l -> row + l/8, chunk position l%8
    const int prow[3] = {R, diag0 ? C2 : C1, C2};  // the rows (in units of 128) of the p-th panel of a stage
    int voffA[NPL][LPP], voffG[NPL][LPP];
    uint32_t ldsoff[NPL][LPP];
#pragma unroll
    for (int p = 0; p < NPL; ++p)
#pragma unroll
        for (int j = 0; j < LPP; ++j) {
            const int row0 = (LPP * wave + j) * 8, row = row0 + (lane >> 3);
            const int cg = (lane & 7) ^ swz(row);
            voffA[p][j] = ((prow[p] * GB + row) * d_in + cg * 8) * 2;
            voffG[p][j] = ((prow[p] * GB + row) * d_out + cg * 8) * 2;
            ldsoff[p][j] = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint16_t*)&ring[p * PANEL + row0 * GU_K];
        }
    int ibuf = 0;
    auto issue = [&](int st) {
        // past the last chunk the loads still go out (the wait counts stay uniform): they read the last chunk again, into
        // a slot that nobody multiplies any more
        const int stc = st < nch ? st : nch - 1;
        const bool isA = stc < nchA;
        // (rotating the chunk order by the example index, which pays in gram_dma_kernel, costs 1-2 % here: the units of an
        // example need their panels at the same time, and any order serves that)
        const int soff = __builtin_amdgcn_readfirstlane((isA ? stc : stc - nchA) * GU_K * 2);
        auto run = [&](const gram_i32x4& rs, const int (&voff)[NPL][LPP]) {  // (the choice of the source stays outside the run of loads)
#pragma unroll
            for (int p = 0; p < NPL; ++p)
#pragma unroll
                for (int j = 0; j < LPP; ++j)
                    gram_dma16<false>(rs, __builtin_amdgcn_readfirstlane(ldsoff[p][j] + ibuf * (STAGE * 2)), voff[p][j], soff);
        };
        if (isA) run(rA, voffA);
        else run(rG, voffG);
        ibuf = ibuf + 1 == GU_NS ? 0 : ibuf + 1;
    };
    // operand of the 16x16x32 MFMA: lane l holds k = 8*(l/16) .. +7 of row l%16 of its 16-row tile, i.e. 16-byte chunk
    // 4*kk + l/16 of that row; a wave's 64 x 64 quadrant is 4 x 4 such tiles.  The 64-row strip its row fragments come
    // from is (panel rslot, half rhalf), that of its column fragments (cslot, chalf).  In a diagonal block the four strips
    // of the two panels are numbered 0..3; wave w < 6 has the quadrant (strip SR[w], strip SC[w]) above the diagonal,
    // waves 6 and 7 the diagonal quadrants of the strips (0, 1) and (2, 3): their "row" fragments are strip SR and their
    // "column" fragments strip SC, each multiplied with itself.
    int rslot = 0, rhalf = wr, cslot = cell == 0 ? (diag0 ? 0 : 1) : NPL - 1, chalf = wc;
    if (BLK) {
        const int sr = (0x20211000u >> (4 * wave)) & 15, sc = (0x31332321u >> (4 * wave)) & 15;
        rslot = sr >> 1, rhalf = sr & 1, cslot = sc >> 1, chalf = sc & 1;
    }
    int fr[4], fc[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int r = rhalf * 64 + u * 16 + (lane & 15), c = chalf * 64 + u * 16 + (lane & 15);
        fr[u] = r * GU_K + (((lane >> 4) ^ swz(r)) << 3) + rslot * PANEL;
        fc[u] = c * GU_K + (((lane >> 4) ^ swz(c)) << 3) + cslot * PANEL;
    }

#pragma unroll
    for (int st = 0; st < GU_NS - 1; ++st) issue(st);
    int cbuf = 0, s_next = GU_NS - 1;
    // A stage is two k steps of 32.  Fragment reads run half a stage ahead of the multiplies and across the barrier:
    // behind the barrier that publishes stage s the wave first asks for the fragments of (s, k step 0), then multiplies
    // those of (s-1, k step 1), which it already holds, asks for (s, k step 1) into the registers just freed, and
    // multiplies (s, k step 0).  All eight waves come out of the barrier together; without the step held over, the
    // matrix pipes would idle behind every barrier until the LDS has served the first reads of all of them.
    struct Frags {
        bf16x8_t a[4], b[4];
    };
    struct Acc {
        f32x4_t t[4][4], t2[4][4];  // t2: the second diagonal quadrant of MODE 3 (never touched otherwise)
    };
    auto read_frags = [&](Frags& f, int kk) {
        const uint16_t* st = ring + cbuf * STAGE;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int xr = fr[u] ^ ((4 * kk) << 3), xc = fc[u] ^ ((4 * kk) << 3);
            f.a[u] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(st + xr));
            f.b[u] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(st + xc));
        }
    };
    // MODE 0: a wave with nothing to multiply (it still fills its share of every stage), 1: a full quadrant, 2: a diagonal
    // quadrant (tiles below its diagonal mirror those above and are skipped), 3: two diagonal quadrants.  The mode is fixed
    // per wave, so the loops exist once per mode, each with accumulators of its own and the final sum inside: a choice
    // inside the loop body would merge the accumulators of its arms after every stage, which costs the register allocator
    // more than it has.
    auto all_stages = [&](auto mode_tag) -> float {
        constexpr int MODE = decltype(mode_tag)::value;
        Acc accA, accG;
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int r = 0; r < 4; ++r) accA.t[a][b][r] = accG.t[a][b][r] = accA.t2[a][b][r] = accG.t2[a][b][r] = 0.f;
        auto multiply = [&](Acc& acc, const Frags& f) {
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                for (int nt = 0; nt < 4; ++nt) {
                    if (MODE == 3) {
                        if (mt <= nt) {
                            acc.t[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.a[mt], f.a[nt], acc.t[mt][nt], 0, 0, 0);
                            acc.t2[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.b[mt], f.b[nt], acc.t2[mt][nt], 0, 0, 0);
                        }
                    } else if (!(MODE == 2 && mt > nt)) {
                        acc.t[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.a[mt], f.b[nt], acc.t[mt][nt], 0, 0, 0);
                    }
                }
        };
        Frags X, Y;
        auto stage = [&](Acc& acc_prev, Acc& acc_cur, auto first_tag) {
            // my loads of this chunk have landed (later chunks may be in flight); after the barrier everyone's have,
            // and everyone is done reading the chunk before this one, whose slot the newest chunk overwrites
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"((GU_NS - 2) * LPS) : "memory");
            __syncthreads();
            issue(s_next++);
            if (MODE != 0) {
                read_frags(X, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (!decltype(first_tag)::value) multiply(acc_prev, Y);
                __builtin_amdgcn_sched_barrier(0);
                read_frags(Y, 1);
                __builtin_amdgcn_sched_barrier(0);
                multiply(acc_cur, X);
                __builtin_amdgcn_sched_barrier(0);
            }
            cbuf = cbuf + 1 == GU_NS ? 0 : cbuf + 1;
        };
        stage(accA, accA, std::true_type{});
        for (int s = 1; s < nchA; ++s) stage(accA, accA, std::false_type{});
        stage(accA, accG, std::false_type{});  // the first chunk of G: the step held over still belongs to A
        for (int s = nchA + 1; s < nch; ++s) stage(accG, accG, std::false_type{});
        if (MODE != 0) multiply(accG, Y);
        float sum = 0.f;
        if (MODE != 0) {
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        // in a diagonal quadrant the tiles above the diagonal stand for their mirror images too; skipped tiles hold zeros
                        const float w = (MODE >= 2 && a < b) ? 2.f : 1.f;
                        sum += w * ((accA.t[a][b][r] + bias_term) * accG.t[a][b][r]);
                        if (MODE == 3) sum += w * ((accA.t2[a][b][r] + bias_term) * accG.t2[a][b][r]);
                    }
        }
        return sum;
    };
    float sum;
    if (!active) sum = all_stages(std::integral_constant<int, 0>{});
    else if (twodiag) sum = all_stages(std::integral_constant<int, 3>{});
    else if (diagw) sum = all_stages(std::integral_constant<int, 2>{});
    else sum = all_stages(std::integral_constant<int, 1>{});
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // nothing may still be writing LDS past this point
    // a quadrant off the diagonal of the plane counts twice (its mirror image is never formed): every quadrant of a cell off
    // the diagonal, the upper-right quadrant of a diagonal cell, and the six quadrants above the diagonal of a diagonal block
    float weight;
    if (BLK) weight = twodiag ? 1.f : 2.f;
    else weight = !active ? 0.f : ((cell == 0 && diag0) ? (wr == wc ? 1.f : 2.f) : 2.f);
    return sum * weight;
}

// out: partials [B][n_layers * n_units], stored.  Workgroup id g -> XCD g % 8; (layer, example) u = (g / 8 / n_units) * 8 + g % 8,
// unit = (g / 8) % n_units: the units of one example share an XCD, so that each panel comes from HBM once.
__global__ __launch_bounds__(512, 1) void gram_units_kernel(GramBatch gb, GramUnits gu, int T, int d_in, int d_out, int has_bias,
                                                            float* __restrict__ out) {
    __shared__ __attribute__((aligned(16))) uint16_t ring[GU_LDS];
    const int slot = blockIdx.x >> 3;
    const int u = (slot / gu.n_units) * 8 + (blockIdx.x & 7);
    const int unit = slot % gu.n_units;
    if (u >= gb.n_layers * gb.B) return;
    const int layer = u / gb.B, i = u - layer * gb.B;
    const uint32_t rc = gu.rc[unit];
    const int R = rc & 255, C1 = (rc >> 8) & 255, C2 = (rc >> 16) & 255;
    const bool blk = (rc >> 24) & 1;
    const uint16_t* A = gb.A[layer] + (size_t)i * T * d_in;
    const uint16_t* G = gb.G[layer] + (size_t)i * T * d_out;
    const float bias_term = has_bias ? 1.f : 0.f;
    const int npl = 1 + (C1 != R ? 1 : 0) + (C2 != 255 ? 1 : 0);
    float s;
    if (blk) s = gram_unit_ring<2, true>(A, G, T, d_in, d_out, R, C1, C2, bias_term, ring);
    else if (npl == 3) s = gram_unit_ring<3, false>(A, G, T, d_in, d_out, R, C1, C2, bias_term, ring);
    else if (npl == 2) s = gram_unit_ring<2, false>(A, G, T, d_in, d_out, R, C1, C2, bias_term, ring);
    else s = gram_unit_ring<1, false>(A, G, T, d_in, d_out, R, C1, C2, bias_term, ring);
    __syncthreads();  // the ring is free: its first floats serve the reduction
    const float tot = dp_block_sum<512>(s, reinterpret_cast<float*>(&ring[0]));
    if (threadIdx.x == 0) out[((size_t)i * gb.n_layers + layer) * gu.n_units + unit] = tot;
}

// ------------------------------------------------------------------------------------------------
// T <= 32 (the output projection of a tied table has 20 rows per example and a 30K-wide input): one 32 x 32 Gram tile
// per operand, so the 128-row kernels above would spend their time on empty rows.  One workgroup per example, the
// contraction split over the 8 waves in chunks of 128 columns; fragments come straight from global memory (lane =
// (row, half) reads 128 contiguous bytes per chunk, the two lanes of a row 256; the MFMA's k slots take the same
// columns for both operands of X X^T, which are the same registers).  The waves' accumulators meet in LDS.
// Bound: HBM, B*T*(d_in+d_out)*2 bytes read once.
// ------------------------------------------------------------------------------------------------
constexpr int GS_WAVES = 8;   // waves per workgroup
constexpr int GS_CHUNK = 128;  // columns per wave and step (each lane: 64 columns = 128 contiguous bytes)

__device__ __forceinline__ void gram_small_load(const uint16_t* __restrict__ row, bool valid, int d, int kb, int half,
                                                gram_i32x4 f[8]) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int k = kb + half * 64 + j * 8;  // widths are multiples of 8: a fragment lies inside the row or outside
        if (valid && k < d) f[j] = __builtin_nontemporal_load(reinterpret_cast<const gram_i32x4*>(row + k));  // read once
        else f[j] = gram_i32x4{0, 0, 0, 0};
    }
}

__device__ __forceinline__ void gram_small_mfma(const gram_i32x4 f[8], f32x16_t& acc) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const bf16x8_t x = __builtin_bit_cast(bf16x8_t, f[j]);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, x, acc, 0, 0, 0);
    }
}

// The loads of the next step are issued before the MFMAs of the current one (the kernel lives on bytes in flight):
// two register sets take turns.
__device__ __forceinline__ void gram_small_accumulate(const uint16_t* __restrict__ row, bool valid, int d, int wave, int half,
                                                      f32x16_t& acc) {
    constexpr int STEP = GS_WAVES * GS_CHUNK;
    gram_i32x4 f0[8], f1[8];
    int kb = wave * GS_CHUNK;
    if (kb >= d) return;
    gram_small_load(row, valid, d, kb, half, f0);
    while (true) {
        if (kb + STEP < d) gram_small_load(row, valid, d, kb + STEP, half, f1);
        gram_small_mfma(f0, acc);
        kb += STEP;
        if (kb >= d) break;
        if (kb + STEP < d) gram_small_load(row, valid, d, kb + STEP, half, f0);
        gram_small_mfma(f1, acc);
        kb += STEP;
        if (kb >= d) break;
    }
}

__global__ __launch_bounds__(64 * GS_WAVES, 4) void gram_small_kernel(const uint16_t* __restrict__ A, const uint16_t* __restrict__ G,
                                                                   int T, int d_in, int d_out, int has_bias,
                                                                   float* __restrict__ out) {
    __shared__ float part[GS_WAVES / 2][2][16][64];
    __shared__ float wred[GS_WAVES];
    const int i = blockIdx.x;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r32 = lane & 31, half = lane >> 5;
    const bool valid = r32 < T;  // rows from T on stay zero in both Gram tiles
    const size_t row = (size_t)i * T + (valid ? r32 : 0);
    f32x16_t accA, accG;
#pragma unroll
    for (int r = 0; r < 16; ++r) accA[r] = 0.f;
    gram_small_accumulate(A + row * d_in, valid, d_in, wave, half, accA);
#pragma unroll
    for (int r = 0; r < 16; ++r) accG[r] = 0.f;
    gram_small_accumulate(G + row * d_out, valid, d_out, wave, half, accG);
    // waves w + 4 hand their tiles to waves w, then the four sums meet
    constexpr int HW = GS_WAVES / 2;
    if (wave >= HW) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            part[wave - HW][0][r][lane] = accA[r];
            part[wave - HW][1][r][lane] = accG[r];
        }
    }
    __syncthreads();
    if (wave < HW) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            accA[r] += part[wave][0][r][lane];
            accG[r] += part[wave][1][r][lane];
        }
    }
    __syncthreads();
    if (wave < HW) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            part[wave][0][r][lane] = accA[r];
            part[wave][1][r][lane] = accG[r];
        }
    }
    __syncthreads();
    const float bias_term = has_bias ? 1.f : 0.f;
    float s = 0.f;
#pragma unroll
    for (int q = 0; q < 16 / GS_WAVES; ++q) {  // wave w finishes accumulator registers 2w, 2w+1; partial tiles added in index order
        const int r = wave * (16 / GS_WAVES) + q;
        const float a = ((part[0][0][r][lane] + part[1][0][r][lane]) + part[2][0][r][lane]) + part[3][0][r][lane];
        const float g = ((part[0][1][r][lane] + part[1][1][r][lane]) + part[2][1][r][lane]) + part[3][1][r][lane];
        s += (a + bias_term) * g;
    }
    const float tot = dp_block_sum<64 * GS_WAVES>(s, wred);
    if (threadIdx.x == 0) out[i] += tot;
}

// The same tile fed like gram_dma_kernel (widths multiples of 64): 128-byte row segments of the 32 rows go straight
// into a ring of 4 KiB stages (one 16-byte-per-lane load per wave and stage, coalesced over 8 rows), and wave w takes
// k step w of every stage: one fragment read and one MFMA per wave and stage.  Loading fragments from global memory
// directly, as the kernel above does, touches 16 bytes of 40 different lines per instruction and was bound by L1/L2
// traffic (1.9 TB/s); here every line crosses once.  NS - 1 stages in flight per workgroup, two workgroups per CU.
template <int NS>
__global__ __launch_bounds__(256, 2) void gram_small_dma_kernel(const uint16_t* __restrict__ A, const uint16_t* __restrict__ G,
                                                                int T, int d_in, int d_out, int has_bias,
                                                                float* __restrict__ out) {
    constexpr int GDK = 64, ROWS = 32, STAGE = ROWS * GDK, CPR = 8, RPI = 8;  // 4 loads fill a stage: one per wave
    static_assert(NS * STAGE * 2 >= 4 * 2 * 16 * 64 * 4, "the ring doubles as the reduction buffer");
    __shared__ __attribute__((aligned(16))) uint16_t ring[NS][STAGE];
    __shared__ float wred[4];
    const int i = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nchA = d_in / GDK, nch = nchA + d_out / GDK;
    auto swz = [](int r) { return (r >> 1) & 7; };  // chunk position c of row r holds global chunk c ^ swz(r)
    // rows >= T lie outside the example's byte range and read as zero
    const gram_i32x4 rA = gram_rsrc(A + (size_t)i * T * d_in, (uint32_t)((size_t)T * d_in * 2));
    const gram_i32x4 rG = gram_rsrc(G + (size_t)i * T * d_out, (uint32_t)((size_t)T * d_out * 2));
    const int lrow = wave * RPI + lane / CPR;
    const int cg = (lane % CPR) ^ swz(lrow);
    const int voffA = (lrow * d_in + cg * 8) * 2, voffG = (lrow * d_out + cg * 8) * 2;
    const uint32_t ldsoff = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint16_t*)&ring[0][wave * RPI * GDK];
    int ibuf = 0;  // buffer of the next stage to issue
    auto issue = [&](int st) {
        const bool isA = st < nchA;
        const int soff = __builtin_amdgcn_readfirstlane((isA ? st : st - nchA) * GDK * 2);
        const uint32_t dst = __builtin_amdgcn_readfirstlane(ldsoff + ibuf * (STAGE * 2));
        if (isA) gram_dma16<true>(rA, dst, voffA, soff);
        else if (st >= nch) gram_dma16<true>(rG, dst, voffG, 0x7FFFFFF0);  // past the end: reads zeros, keeps the load count uniform
        else gram_dma16<true>(rG, dst, voffG, soff);
        ibuf = ibuf + 1 == NS ? 0 : ibuf + 1;
    };
    const int r = lane & 31;
    const int fpos = r * GDK + (((2 * wave + (lane >> 5)) ^ swz(r)) << 3);  // this wave's k step of a stage
    f32x16_t accA, accG;
#pragma unroll
    for (int q = 0; q < 16; ++q) accA[q] = accG[q] = 0.f;
#pragma unroll
    for (int st = 0; st < NS - 1; ++st) issue(st);
    int cbuf = 0, s = 0;
    auto phase = [&](int end, f32x16_t& acc) {
        for (; s < end; ++s) {
            // my load of stage s has landed (later ones may be in flight); after the barrier everyone's have, and
            // everyone is done reading stage s-1, whose buffer the newest stage overwrites
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NS - 2) : "memory");
            __syncthreads();
            issue(s + NS - 1);
            const bf16x8_t x = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(ring[cbuf] + fpos));
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, x, acc, 0, 0, 0);
            cbuf = cbuf + 1 == NS ? 0 : cbuf + 1;
        }
    };
    phase(nchA, accA);
    phase(nch, accG);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // nothing may still be writing LDS when the ring is reused
    __syncthreads();
    float* part = reinterpret_cast<float*>(&ring[0][0]);  // [wave][A|G][register][lane]
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        part[((wave * 2 + 0) * 16 + q) * 64 + lane] = accA[q];
        part[((wave * 2 + 1) * 16 + q) * 64 + lane] = accG[q];
    }
    __syncthreads();
    const float bias_term = has_bias ? 1.f : 0.f;
    float sum = 0.f;
#pragma unroll
    for (int q = 0; q < 4; ++q) {  // wave w finishes accumulator registers 4w .. 4w+3, the waves' partial tiles added in index order
        const int reg = wave * 4 + q;
        float a = 0.f, g = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            a += part[((w * 2 + 0) * 16 + reg) * 64 + lane];
            g += part[((w * 2 + 1) * 16 + reg) * 64 + lane];
        }
        sum += (a + bias_term) * g;
    }
    const float tot = dp_block_sum<256>(sum, wred);
    if (threadIdx.x == 0) out[i] += tot;
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

// The LDS-ring kernel serves one 128 x 128 block per example and widths that are multiples of its row segment.
static bool gram_dma_ok(int T, int d_in, int d_out) {
    return T <= GB && d_in % GK == 0 && d_out % GK == 0 && d_in > 0 && d_out > 0 &&
           (size_t)T * (d_in > d_out ? d_in : d_out) * 2 < (1u << 31);
}

static dp_status gram_dma_launch(dp_ctx* ctx, const GramBatch& gb, int T, int d_in, int d_out, int has_bias, float* out,
                                 double bytes) {
    dp_prof_scope prof(ctx, DP_PROF_GRAM, bytes);
    const dim3 grid((unsigned)((long)gb.n_layers * gb.B)), block(256);
    // 256-byte row segments (two stages of 32 KiB) when the widths allow, else 128-byte segments (four stages of 16 KiB)
    if (d_in % 128 == 0 && d_out % 128 == 0)
        hipLaunchKernelGGL((gram_dma_kernel<128, 2, 2>), grid, block, 0, ctx->stream, gb, T, d_in, d_out, has_bias, out);
    else
        hipLaunchKernelGGL((gram_dma_kernel<64, 4, 2>), grid, block, 0, ctx->stream, gb, T, d_in, d_out, has_bias, out);
    DP_LAUNCH_CHECK(ctx, "gram_dma");
    return DP_OK;
}

// The upper triangle of an nblk x nblk plane of 128 x 128 cells, cut into units.  Panels go two by two: the pair (2I, 2I+1)
// gives the diagonal block (2I, 2I), (2I, 2I+1), (2I+1, 2I+1); two pairs I < J give the four cells of rows 2I, 2I+1 and
// columns 2J, 2J+1, i.e. two row pairs.  With an odd nblk the last panel has no partner: its diagonal cell leads the row
// pair (last, last), (last, 0) - by symmetry (last, r) stands for the cell (r, last) - the cells (r, last) of the other
// rows pair up through the shared panel, (last, r1), (last, r2), and one of them stays alone.
static GramUnits gram_make_units(int nblk) {
    GramUnits gu;
    int n = 0;
    const int npair = nblk / 2, last = nblk - 1;
    for (int I = 0; I < npair; ++I) gu.rc[n++] = (uint32_t)(2 * I) | (uint32_t)(2 * I) << 8 | (uint32_t)(2 * I + 1) << 16 | 1u << 24;
    for (int I = 0; I < npair; ++I)
        for (int J = I + 1; J < npair; ++J)
            for (int r = 2 * I; r < 2 * I + 2; ++r) gu.rc[n++] = (uint32_t)r | (uint32_t)(2 * J) << 8 | (uint32_t)(2 * J + 1) << 16;
    if (nblk & 1) {
        gu.rc[n++] = (uint32_t)last | (uint32_t)last << 8 | (last > 0 ? 0u : 255u) << 16;
        int r = 1;
        for (; r + 1 < last; r += 2) gu.rc[n++] = (uint32_t)last | (uint32_t)r << 8 | (uint32_t)(r + 1) << 16;
        if (r < last) gu.rc[n++] = (uint32_t)r | (uint32_t)last << 8 | 255u << 16;
    }
    gu.n_units = n;
    return gu;
}

// The unit kernel: T up to GU_MAX_BLK cells of 128 rows, widths multiples of its 64-wide chunk.
static bool gram_units_ok(int T, int d_in, int d_out) {
    return T > GB && T <= GB * GU_MAX_BLK && d_in % GU_K == 0 && d_out % GU_K == 0 && d_in > 0 && d_out > 0 &&
           (size_t)T * (d_in > d_out ? d_in : d_out) * 2 < (1u << 31);
}

dp_status dpk_gram_unit_plan(int T, uint32_t* units, int capacity, int* n_units) {
    if (T <= GB || T > GB * GU_MAX_BLK) return DP_ERR_SHAPE;
    const GramUnits gu = gram_make_units((T + GB - 1) / GB);
    if (gu.n_units > capacity) return DP_ERR_WORKSPACE;
    for (int k = 0; k < gu.n_units; ++k) units[k] = gu.rc[k];
    *n_units = gu.n_units;
    return DP_OK;
}

// nl <= GRAM_MAX_BATCH same-shaped layers: partials [B][nl * n_units] through the workspace, added in index order.
static dp_status gram_units_launch(dp_ctx* ctx, const GramBatch& gb, int T, int d_in, int d_out, int has_bias,
                                   float* sqnorms) {
    const GramUnits gu = gram_make_units((T + GB - 1) / GB);
    const long units = (long)gb.n_layers * gb.B;
    const long nwg = (units + 7) / 8 * 8 * gu.n_units;
    if (nwg > 0x7FFFFFFFl) {
        DP_SET_ERR(ctx, "dp_sqnorms_dense: B * T^2 too large for one launch");
        return DP_ERR_SHAPE;
    }
    dp_ws_alloc ws(ctx);
    float* part = ws.get<float>((size_t)units * gu.n_units);
    if (!part) {
        DP_SET_ERR(ctx, "workspace too small for %ld x %d Gram partials", units, gu.n_units);
        return DP_ERR_WORKSPACE;
    }
    {
        dp_prof_scope prof(ctx, DP_PROF_GRAM, 2.0 * (double)gb.B * T * ((double)d_in + d_out) * gb.n_layers);
        hipLaunchKernelGGL(gram_units_kernel, dim3((unsigned)nwg), dim3(512), 0, ctx->stream, gb, gu, T, d_in, d_out,
                           has_bias, part);
    }
    DP_LAUNCH_CHECK(ctx, "gram_units");
    return dpk_finish_partials(ctx, part, gb.B, gu.n_units * gb.n_layers, sqnorms);
}

dp_status dpk_gram_sqnorms_batched(dp_ctx* ctx, int n_layers, const void* const* A, const void* const* G, dp_dtype dt,
                                   int B, int T, int d_in, int d_out, int has_bias, float* sqnorms) {
    if (dt == DP_BF16 && gram_units_ok(T, d_in, d_out)) {
        // enough layers per launch for a few rounds of workgroups, and partials that fit the workspace
        const int nblk = (T + GB - 1) / GB;
        const long npairs = (long)nblk * (nblk + 1) / 2;  // (an upper bound of the units per example)
        int per = GRAM_MAX_BATCH;
        while (per > 1 && ((size_t)per * B * npairs * sizeof(float) > ctx->ws_bytes / 2 ||
                           (long)per * B * npairs > (1l << 22)))
            per /= 2;
        for (int l0 = 0; l0 < n_layers; l0 += per) {
            const int nl = n_layers - l0 < per ? n_layers - l0 : per;
            GramBatch gb;
            for (int l = 0; l < GRAM_MAX_BATCH; ++l) {
                gb.A[l] = (const uint16_t*)A[l0 + (l < nl ? l : 0)];
                gb.G[l] = (const uint16_t*)G[l0 + (l < nl ? l : 0)];
                gb.G2[l] = gb.G3[l] = gb.G[l];
            }
            gb.n_layers = nl;
            gb.n_out = 1;
            gb.B = B;
            dp_status st = gram_units_launch(ctx, gb, T, d_in, d_out, has_bias, sqnorms);
            if (st != DP_OK) return st;
        }
        return DP_OK;
    }
    if (dt != DP_BF16 || !gram_dma_ok(T, d_in, d_out) || (long)B * GRAM_MAX_BATCH > 0x7FFFFFFFl) {
        for (int l = 0; l < n_layers; ++l) {
            dp_status st = dpk_gram_sqnorms(ctx, A[l], G[l], dt, B, T, d_in, d_out, has_bias, sqnorms);
            if (st != DP_OK) return st;
        }
        return DP_OK;
    }
    for (int l0 = 0; l0 < n_layers; l0 += GRAM_MAX_BATCH) {
        const int nl = n_layers - l0 < GRAM_MAX_BATCH ? n_layers - l0 : GRAM_MAX_BATCH;
        GramBatch gb;
        for (int l = 0; l < GRAM_MAX_BATCH; ++l) {
            gb.A[l] = (const uint16_t*)A[l0 + (l < nl ? l : 0)];
            gb.G[l] = (const uint16_t*)G[l0 + (l < nl ? l : 0)];
            gb.G2[l] = gb.G3[l] = gb.G[l];
        }
        gb.n_layers = nl;
        gb.n_out = 1;
        gb.B = B;
        const double bytes = 2.0 * (double)B * T * ((double)d_in + d_out) * nl;
        if (nl == 1) {
            dp_status st = gram_dma_launch(ctx, gb, T, d_in, d_out, has_bias, sqnorms, bytes);
            if (st != DP_OK) return st;
            continue;
        }
        dp_ws_alloc ws(ctx);
        float* part = ws.get<float>((size_t)B * nl);
        if (!part) {
            DP_SET_ERR(ctx, "workspace too small for %d x %d norm partials", B, nl);
            return DP_ERR_WORKSPACE;
        }
        dp_status st = gram_dma_launch(ctx, gb, T, d_in, d_out, has_bias, part, bytes);
        if (st != DP_OK) return st;
        st = dpk_finish_partials(ctx, part, B, nl, sqnorms);   // layers added in index order
        if (st != DP_OK) return st;
    }
    return DP_OK;
}

// n_groups groups of n_out (2 or 3) same-shaped layers, the layers of a group sharing their input A[g]; G is
// group-major: G[g * n_out + j].
dp_status dpk_gram_sqnorms_shared(dp_ctx* ctx, int n_groups, const void* const* A, int n_out, const void* const* G,
                                  dp_dtype dt, int B, int T, int d_in, int d_out, int has_bias, float* sqnorms) {
    if (dt != DP_BF16 || n_out < 2 || n_out > 3 || !gram_dma_ok(T, d_in, d_out) ||
        (long)B * GRAM_MAX_BATCH > 0x7FFFFFFFl) {
        for (int g = 0; g < n_groups; ++g)
            for (int j = 0; j < n_out; ++j) {
                dp_status st = dpk_gram_sqnorms(ctx, A[g], G[(size_t)g * n_out + j], dt, B, T, d_in, d_out, has_bias, sqnorms);
                if (st != DP_OK) return st;
            }
        return DP_OK;
    }
    for (int g0 = 0; g0 < n_groups; g0 += GRAM_MAX_BATCH) {
        const int ng = n_groups - g0 < GRAM_MAX_BATCH ? n_groups - g0 : GRAM_MAX_BATCH;
        GramBatch gb;
        for (int l = 0; l < GRAM_MAX_BATCH; ++l) {
            const size_t g = (size_t)g0 + (l < ng ? l : 0);
            gb.A[l] = (const uint16_t*)A[g];
            gb.G[l] = (const uint16_t*)G[g * n_out];
            gb.G2[l] = (const uint16_t*)G[g * n_out + 1];
            gb.G3[l] = (const uint16_t*)G[g * n_out + (n_out > 2 ? 2 : 1)];
        }
        gb.n_layers = ng;
        gb.n_out = n_out;
        gb.B = B;
        const double bytes = 2.0 * (double)B * T * ((double)d_in + (double)n_out * d_out) * ng;
        if (ng == 1) {
            dp_status st = gram_dma_launch(ctx, gb, T, d_in, d_out, has_bias, sqnorms, bytes);
            if (st != DP_OK) return st;
            continue;
        }
        dp_ws_alloc ws(ctx);
        float* part = ws.get<float>((size_t)B * ng);
        if (!part) {
            DP_SET_ERR(ctx, "workspace too small for %d x %d norm partials", B, ng);
            return DP_ERR_WORKSPACE;
        }
        dp_status st = gram_dma_launch(ctx, gb, T, d_in, d_out, has_bias, part, bytes);
        if (st != DP_OK) return st;
        st = dpk_finish_partials(ctx, part, B, ng, sqnorms);
        if (st != DP_OK) return st;
    }
    return DP_OK;
}

dp_status dpk_gram_sqnorms(dp_ctx* ctx, const void* A, const void* G, dp_dtype dt, int B, int T, int d_in, int d_out,
                           int has_bias, float* sqnorms) {
    if (dt == DP_F32) {
        hipLaunchKernelGGL(gram_f32_kernel, dim3(B), dim3(256), 0, ctx->stream, (const float*)A, (const float*)G, T,
                           d_in, d_out, has_bias, sqnorms);
        DP_LAUNCH_CHECK(ctx, "gram_f32");
        return DP_OK;
    }
    if (T <= 32 && d_in % 64 == 0 && d_out % 64 == 0 && 64l * (d_in > d_out ? d_in : d_out) < (1l << 31)) {
        dp_prof_scope prof(ctx, DP_PROF_GRAM, 2.0 * (double)B * T * ((double)d_in + d_out));
        hipLaunchKernelGGL((gram_small_dma_kernel<16>), dim3(B), dim3(256), 0, ctx->stream, (const uint16_t*)A,
                           (const uint16_t*)G, T, d_in, d_out, has_bias, sqnorms);
        DP_LAUNCH_CHECK(ctx, "gram_small_dma");
        return DP_OK;
    }
    if (T <= 32) {
        dp_prof_scope prof(ctx, DP_PROF_GRAM, 2.0 * (double)B * T * ((double)d_in + d_out));
        hipLaunchKernelGGL(gram_small_kernel, dim3(B), dim3(64 * GS_WAVES), 0, ctx->stream, (const uint16_t*)A, (const uint16_t*)G, T,
                           d_in, d_out, has_bias, sqnorms);
        DP_LAUNCH_CHECK(ctx, "gram_small");
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
    if (gram_dma_ok(T, d_in, d_out) || gram_units_ok(T, d_in, d_out)) {
        GramBatch gb;
        for (int l = 0; l < GRAM_MAX_BATCH; ++l) {
            gb.A[l] = (const uint16_t*)A;
            gb.G[l] = (const uint16_t*)G;
            gb.G2[l] = gb.G3[l] = gb.G[l];
        }
        gb.n_layers = 1;
        gb.n_out = 1;
        gb.B = B;
        if (T > GB) return gram_units_launch(ctx, gb, T, d_in, d_out, has_bias, sqnorms);
        return gram_dma_launch(ctx, gb, T, d_in, d_out, has_bias, sqnorms, bytes);
    }
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
