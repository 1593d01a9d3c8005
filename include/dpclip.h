/*
 * dpclip.h - C ABI of the MI355X (gfx950) DP-SGD hot path: per-example squared gradient norms,
 * clip-weighted gradient sums accumulated over micro-batches, and the Gaussian-noise + Adam update
 * with decoupled weight decay ("Large-Scale Differentially Private BERT", Algorithm 1).
 *
 * One training step, in the notation of Algorithm 1 (g_t line through theta_t line):
 *
 *     g_t     = ( N(0, sigma^2 C^2 I) + sum_{x_j in B_t} clip(grad L(theta; x_j), C) ) / |B_t|
 *     m_t     = beta1 m_{t-1} + (1 - beta1) g_t          v_t = beta2 v_{t-1} + (1 - beta2) g_t^2
 *     mhat_t  = m_t / (1 - beta1^t)                      vhat_t = v_t / (1 - beta2^t)
 *     theta_t = theta_{t-1} - eta_t ( mhat_t / (sqrt(vhat_t) + xi) + lambda theta_{t-1} )
 *
 * with clip(g, C) = g * min(1, C / ||g||_2), the norm taken over ALL parameters of one example's
 * gradient.  The mega-batch B_t is processed as micro-batches (Section 5.3, gradient accumulation):
 * for each micro-batch the caller runs pass 1 (dp_sqnorms_* over every layer, "+=" into sqnorms[B]),
 * then pass 2 (dp_clip_accumulate_* over every layer, "+=" into the fp32 sum buffers), and after the
 * last micro-batch one dp_noise_adamw over the flat parameter space.
 *
 * Per-example gradients of the weight tensors are never materialised (the one exception is optional and small:
 * dp_sqnorms_layernorm_keep writes the 2 d numbers of a LayerNorm per example).  For a dense layer y = xW + b with inputs A_i [T, d_in]
 * and output gradients G_i [T, d_out] of example i (the outer-product form of the fully connected
 * layer's gradient, Section 4.3) the example's weight gradient is A_i^T G_i and its bias gradient is
 * sum_t G_i[t, :].
 *
 * Conventions
 *   - Every pointer except dp_ctx* and the out-parameters of dp_create / dp_choose_path is a DEVICE
 *     pointer owned by the caller.  The library neither frees nor keeps it beyond the completion of the
 *     call's work on the context's stream.
 *   - All tensors are dense row-major.  A, Xhat: [B, T, d_in|d];  G: [B, T, d_out|d];  ids: int32 [B, T];
 *     weight-shaped sums: [d_in, d_out];  embedding sums: [V, d].  sqnorms, sums, params, m, v: fp32.
 *   - dtype selects the element type of A / Xhat / G: DP_F32 (4-byte aligned) or DP_BF16 (16-byte aligned
 *     pointers and d_in, d_out, d multiples of 8).  Accumulation is always fp32.
 *   - Calls are asynchronous on the context's stream and return argument and launch errors at once.
 *     Errors found on the device (a token id outside [0, V)) are returned by the next dp_sync.
 *   - Results are deterministic: the same call sequence on the same inputs gives the same bits.
 *   - The step's entry points (norms, clip factors, clip-weighted sums, the update, dp_zero_f32) only launch kernels
 *     on the context's stream: no allocation, no memory-set or copy command, no wait for the device.  A caller may
 *     therefore record them into a HIP graph on that stream (profiling off) and replay it; replays give the bits of
 *     the eager calls.  dp_create, dp_destroy, dp_sync and the dp_profile_* calls do wait and must stay outside.
 *   - No entry point prints, throws or exits.  A context must be used by one host thread at a time.
 */
#ifndef DPCLIP_H
#define DPCLIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dp_ctx dp_ctx; /* opaque: stream, workspace, device error word */

typedef enum { DP_F32 = 0, DP_BF16 = 1 } dp_dtype;

/* How the dense weight-gradient norm is evaluated (see dp_sqnorms_dense). */
typedef enum { DP_PATH_AUTO = 0, DP_PATH_GRAM = 1, DP_PATH_MATERIALISE = 2 } dp_path;

typedef enum {
    DP_OK = 0,
    DP_ERR_NULL = -1,      /* a required pointer is NULL */
    DP_ERR_SHAPE = -2,     /* a size is negative, or not a multiple the dtype requires */
    DP_ERR_DTYPE = -3,     /* unknown dp_dtype / dp_path value */
    DP_ERR_ALIGN = -4,     /* pointer alignment */
    DP_ERR_VALUE = -5,     /* C <= 0, sigma < 0, batch_size == 0, step == 0, beta outside [0,1), eps < 0 ...; from dp_sync: a
                              per-example squared norm that pass 2 read was NaN or had overflowed fp32 */
    DP_ERR_INDEX = -6,     /* a token id outside [0, V) was met on the device (reported by dp_sync) */
    DP_ERR_WORKSPACE = -7, /* the context's workspace is too small for this call */
    DP_ERR_HIP = -8        /* a HIP runtime call failed; dp_last_error has the text */
} dp_status;

/* Create a context bound to `hip_stream` (a hipStream_t, borrowed; NULL = the null stream) on the current
 * device, with a device workspace of `workspace_bytes` (0 = 512 MiB) for clip factors, split-reduction
 * partials and sort buffers.  *out is set only on DP_OK. */
dp_status dp_create(dp_ctx** out, void* hip_stream, size_t workspace_bytes);
/* Synchronise the stream, then free the workspace and the context. */
dp_status dp_destroy(dp_ctx* ctx);
/* hipStreamSynchronize, then fetch-and-clear the device error word: DP_OK, DP_ERR_INDEX (a token id outside
 * [0, V)), DP_ERR_VALUE (a non-finite squared norm met by pass 2; DP_ERR_INDEX wins if both occurred) or DP_ERR_HIP. */
dp_status dp_sync(dp_ctx* ctx);
const char* dp_status_str(dp_status s);
/* Text of the last error of this context; static storage inside the context. */
const char* dp_last_error(const dp_ctx* ctx);

/* ---------------------------------------------------------------------------------------------------
 * Pass 1: per-example squared norms.  Each call ADDS one layer's contribution to sqnorms[i], i < B.
 * The caller zeroes sqnorms once per micro-batch (dp_zero_f32) and calls every layer on one stream;
 * the sum over layers is the squared global norm that clip() of Algorithm 1 needs.
 * B == 0 or T == 0 is a no-op.
 * ------------------------------------------------------------------------------------------------- */

/* Dense layer: sqnorms[i] += ||A_i^T G_i||_F^2  (+ ||sum_t G_i[t,:]||^2 if has_bias).
 * DP_PATH_GRAM evaluates sum_{t,s} (a_t.a_s)(g_t.g_s) from the two T x T Gram matrices;
 * DP_PATH_MATERIALISE forms A_i^T G_i tile by tile and sums the squares; DP_PATH_AUTO picks by
 * dp_choose_path.  Both give the same value up to fp32 rounding order. */
dp_status dp_sqnorms_dense(dp_ctx* ctx, const void* A, const void* G, dp_dtype dtype, int B, int T, int d_in,
                           int d_out, int has_bias, dp_path path, float* sqnorms);

/* n_layers dense layers of one shape in one call: the result is that of n_layers calls of dp_sqnorms_dense
 * with the same arguments (each layer's norms added to sqnorms[i], layers in index order).  On the Gram path
 * with widths that are multiples of 64 the layers share launches of up to 16 layers, which keeps the memory
 * pipeline full across examples; their per-layer norms (for T > 128: per layer and unit of two or three 128 x 128 cells of the T x T plane) pass
 * through the library workspace and are added in a fixed order (DP_ERR_WORKSPACE if they do not fit).
 * A, G are HOST arrays of n_layers device pointers, read during the call only. */
dp_status dp_sqnorms_dense_batched(dp_ctx* ctx, int n_layers, const void* const* A, const void* const* G, dp_dtype dtype,
                                   int B, int T, int d_in, int d_out, int has_bias, dp_path path, float* sqnorms);

/* Layers that share their input (the query, key and value projections of an attention block read the same
 * activations): n_groups groups of n_out same-shaped layers, group g's layers having input A[g] and output
 * gradients G[g * n_out + j], j < n_out.  The result is that of n_groups * n_out calls of dp_sqnorms_dense (every
 * layer with its own bias if has_bias).  Because sum_j <A A^T (+1), G_j G_j^T> = <A A^T (+1), sum_j G_j G_j^T>, the
 * Gram path (T <= 128, widths multiples of 64, n_out 2 or 3) forms A A^T once per group and reads A once: a
 * third fewer bytes and matrix operations for a query/key/value group.  Other shapes are served layer by layer.
 * A (n_groups entries) and G (n_groups * n_out entries) are HOST arrays of device pointers, read during the call. */
dp_status dp_sqnorms_dense_shared(dp_ctx* ctx, int n_groups, const void* const* A, int n_out, const void* const* G,
                                  dp_dtype dtype, int B, int T, int d_in, int d_out, int has_bias, float* sqnorms);

/* LayerNorm y = gamma * xhat + beta, Xhat = the NORMALISED activations:
 * sqnorms[i] += sum_j (sum_t G[i,t,j] Xhat[i,t,j])^2 + sum_j (sum_t G[i,t,j])^2. */
dp_status dp_sqnorms_layernorm(dp_ctx* ctx, const void* Xhat, const void* G, dp_dtype dtype, int B, int T, int d,
                               float* sqnorms);

/* n_layers LayerNorms of one shape in one call: the result of n_layers calls of dp_sqnorms_layernorm (layers added
 * in index order).  Up to 16 layers share a launch; their per-example partial norms pass through the library
 * workspace (DP_ERR_WORKSPACE if they do not fit).  Xhat, G: HOST arrays of n_layers device pointers, read during the
 * call only. */
dp_status dp_sqnorms_layernorm_batched(dp_ctx* ctx, int n_layers, const void* const* Xhat, const void* const* G,
                                       dp_dtype dtype, int B, int T, int d, float* sqnorms);

/* Embedding lookup y_t = E[ids_t] (Section 4.3 names the word-piece, positional and token-type tables):
 * sqnorms[i] += sum_v || sum_{t: ids[i,t] = v} G[i,t,:] ||^2.
 * distinct_per_example != 0 promises that no id repeats inside an example (position ids), which
 * reduces the value to ||G_i||_F^2; ids are then only range-checked. */
dp_status dp_sqnorms_embedding(dp_ctx* ctx, const int32_t* ids, const void* G, dp_dtype dtype, int B, int T, int d,
                               int V, int distinct_per_example, float* sqnorms);

/* ---------------------------------------------------------------------------------------------------
 * Pass 2: clip-weighted sums.  With c_i = min(1, C / sqrt(sqnorms[i])) (c_i = 1 where sqnorms[i] == 0),
 * each call ADDS sum_i c_i * (example i's gradient of this layer) to the caller's fp32 sum buffers.
 * Squared norms live in fp32: an example whose gradient norm exceeds about 1.8e19 overflows it.  Such a value (inf, or
 * NaN) has no clip factor: on every path alike the factor is NaN, the sums that example enters become NaN, and the next
 * dp_sync returns DP_ERR_VALUE - nothing is dropped or passed through unclipped silently.  Finite norms up to the
 * fp32 range are handled exactly like any other (the accumulators of the matrix-core path are rescaled by ratios of
 * neighbouring factors, at most 1.8e19 / C, and hold at most B times the largest norm: both inside the fp32 range).
 * The caller zeroes the sum buffers once per mega-batch; repeated calls over micro-batches accumulate.
 * sqnorms must hold the finished pass-1 result of the SAME micro-batch.
 * ------------------------------------------------------------------------------------------------- */

/* sum_W[p,q] += sum_i c_i sum_t A[i,t,p] G[i,t,q];  sum_b[q] += sum_i c_i sum_t G[i,t,q] (sum_b may be NULL).
 * DP_BF16, accumulation in fp32: for T a multiple of 64 and widths >= 256 the operands enter the matrix-core
 * contraction unscaled (exact bf16 products) and the accumulators are rescaled by c_prev / c_next where the
 * example changes; for other shapes the clip factor multiplies G in fp32 and the product is rounded back to
 * bf16 (round-to-nearest-even) before the contraction (relative error of the sum about 1e-3). */
dp_status dp_clip_accumulate_dense(dp_ctx* ctx, const void* A, const void* G, dp_dtype dtype, int B, int T, int d_in,
                                   int d_out, float C, const float* sqnorms, float* sum_W, float* sum_b);

/* dp_clip_accumulate_dense for n_layers independent layers of ONE shape (same dtype, B, T, d_in, d_out, C and
 * sqnorms) in as few launches as possible: the layers' tiles fill the chip together, so the token rows need not
 * be split and no partial sums pass through memory.  A, G, sum_W, sum_b are HOST arrays of n_layers device
 * pointers (sum_b may be NULL, and so may any of its entries); they are read during the call only.
 * The result of each layer is what dp_clip_accumulate_dense gives, up to fp32 summation order. */
dp_status dp_clip_accumulate_dense_batched(dp_ctx* ctx, int n_layers, const void* const* A, const void* const* G,
                                           dp_dtype dtype, int B, int T, int d_in, int d_out, float C,
                                           const float* sqnorms, float* const* sum_W, float* const* sum_b);

/* sum_gamma[j] += sum_i c_i sum_t G[i,t,j] Xhat[i,t,j];  sum_beta[j] += sum_i c_i sum_t G[i,t,j]. */
dp_status dp_clip_accumulate_layernorm(dp_ctx* ctx, const void* Xhat, const void* G, dp_dtype dtype, int B, int T,
                                       int d, float C, const float* sqnorms, float* sum_gamma, float* sum_beta);

/* n_layers LayerNorms of one shape in one call: the result of n_layers calls of dp_clip_accumulate_layernorm, with
 * one evaluation of the clip factors and up to 16 layers per launch.  Xhat, G, sum_gamma, sum_beta: HOST arrays of
 * n_layers device pointers (none NULL), read during the call only. */
dp_status dp_clip_accumulate_layernorm_batched(dp_ctx* ctx, int n_layers, const void* const* Xhat, const void* const* G,
                                               dp_dtype dtype, int B, int T, int d, float C, const float* sqnorms,
                                               float* const* sum_gamma, float* const* sum_beta);

/* LayerNorm gradients are small (2 d numbers per example and layer), so pass 1 can keep them and pass 2 need not read
 * Xhat and G again: dp_sqnorms_layernorm_keep does what dp_sqnorms_layernorm_batched does and also WRITES every
 * example's gradient to grads[l] (device, fp32, [B][2][d]: row 0 the gain gradient sum_t G Xhat, row 1 the offset
 * gradient sum_t G; 16-byte aligned, d a multiple of 4, caller-owned, overwritten);
 * dp_clip_accumulate_layernorm_kept then adds sum_i c_i grads[l][i] to sum_gamma[l] / sum_beta[l] (16-byte aligned),
 * reading 8 d bytes per example instead of 2 T d elements.  Same sums as dp_clip_accumulate_layernorm up to fp32
 * summation order (examples are added in a fixed order).  The caller must not change grads between the two calls
 * of a micro-batch.  All tables are HOST arrays of n_layers device pointers, read during the call only. */
dp_status dp_sqnorms_layernorm_keep(dp_ctx* ctx, int n_layers, const void* const* Xhat, const void* const* G, dp_dtype dtype,
                                    int B, int T, int d, float* sqnorms, float* const* grads);
dp_status dp_clip_accumulate_layernorm_kept(dp_ctx* ctx, int n_layers, float* const* grads, int B, int d, float C,
                                            const float* sqnorms, float* const* sum_gamma, float* const* sum_beta);

/* sum_E[ids[i,t], :] += c_i G[i,t,:] for every token.  Rows are added in ascending (i, t) order per id. */
dp_status dp_clip_accumulate_embedding(dp_ctx* ctx, const int32_t* ids, const void* G, dp_dtype dtype, int B, int T,
                                       int d, int V, float C, const float* sqnorms, float* sum_E);

/* The position-embedding case of dp_clip_accumulate_embedding: ids[i,t] = t for every example, so
 * sum_E[t, :] += sum_i c_i G[i,t,:] for t < T.  No ids, no sort: one weighted sum over the B examples.  Same result as
 * the general entry point up to fp32 summation order.
 * PRECONDITION: the table behind sum_E has at least T rows of width d (T <= the model's maximum position).  The
 * call takes no table height and cannot check this: it writes rows 0 .. T-1 and touches no row from T on, so a
 * table shorter than T rows is overrun.  A caller that cannot guarantee it uses dp_clip_accumulate_embedding with
 * explicit ids and V, which range-checks every id. */
dp_status dp_clip_accumulate_positions(dp_ctx* ctx, const void* G, dp_dtype dtype, int B, int T, int d, float C,
                                       const float* sqnorms, float* sum_E);

/* A table E [V, d] that every example uses twice (tied weights): as the lookup y_t = E[ids_t] of its T tokens
 * (Section 4.3's word-piece table) and as the output projection logits = H E^T of M selected positions (the
 * masked-token head of BERT; the paper does not say whether its model ties the two: these two entry points are the
 * path's form if it does).  E is one parameter, so an example has one gradient for it,
 *     g_i = scatter(ids_i, dY_i) + dL_i^T H_i     [V, d],
 * dY [B,T,d] the gradient of the lookup's output, H [B,M,d] the inputs of the output projection, dL [B,M,V] the
 * gradient of the logits (rows of unused prediction slots are zero), all of `dtype`, row-major, device memory,
 * caller-owned; bf16 needs d and V multiples of 8; with M = 0 H and dL are not read and may be NULL.  Never materialised:
 *     sqnorms[i] += ||scatter||^2 + <dL_i dL_i^T, H_i H_i^T> + 2 sum_{t,m} dL[i,m,ids[i,t]] <dY[i,t,:], H[i,m,:]>
 * (the embedding norm, the dense norm of a layer with input dL and output gradient H, and the cross term between
 * them, which is not small when a predicted token also occurs in the input).  An id outside [0, V) sets the
 * error flag that dp_sync reports, as in dp_sqnorms_embedding. */
dp_status dp_sqnorms_tied_embedding(dp_ctx* ctx, const int32_t* ids, const void* dY, const void* H, const void* dL,
                                    dp_dtype dtype, int B, int T, int M, int d, int V, float* sqnorms);

/* sum_E += sum_i c_i (scatter(ids_i, dY_i) + dL_i^T H_i), sum_E [V, d] fp32 (16-byte aligned for bf16): the work of
 * dp_clip_accumulate_embedding(ids, dY) followed by dp_clip_accumulate_dense(A = dL, G = H, no bias) into the same
 * buffer. */
dp_status dp_clip_accumulate_tied_embedding(dp_ctx* ctx, const int32_t* ids, const void* dY, const void* H,
                                            const void* dL, dp_dtype dtype, int B, int T, int M, int d, int V, float C,
                                            const float* sqnorms, float* sum_E);

/* The clip factors themselves (pass 2 computes them internally; exposed for checks): c[i], i < B. */
dp_status dp_clip_factors(dp_ctx* ctx, const float* sqnorms, int B, float C, float* c);

/* ---------------------------------------------------------------------------------------------------
 * Update (Algorithm 1, g_t line to theta_t line) over the slice [elem_offset, elem_offset + n) of the
 * flat parameter space; params, m, v, sum point at the slice's first element.
 *   g = (sum + sigma*C*z) / batch_size,  z ~ N(0,1) drawn per GLOBAL element index from Philox4x32-10:
 *   element e uses word e%4 of the block with counter (lo32(e/4), hi32(e/4), lo32(step), hi32(step)) and
 *   key (lo32(seed), hi32(seed)); u = ((word >> 9) + 0.5) * 2^-23; Box-Muller on the word pairs (0,1)
 *   and (2,3): even element rho*cos(2 pi u_odd), odd element rho*sin(2 pi u_odd), rho = sqrt(-2 ln u_even).
 *   The noise therefore does not depend on how the caller slices the update.  sigma == 0 draws nothing.
 * batch_size is the mega-batch example count |B_t|; step is t >= 1 (bias correction and RNG counter);
 * eps is xi (the paper sets 1e-11), added outside the square root; weight decay multiplies theta_{t-1}.
 * zero_sum != 0 also clears `sum` for the next mega-batch.
 * ------------------------------------------------------------------------------------------------- */
dp_status dp_noise_adamw(dp_ctx* ctx, float* params, float* m, float* v, float* sum, uint64_t n,
                         uint64_t elem_offset, float sigma, float C, uint64_t seed, uint64_t step,
                         uint64_t batch_size, float lr, float beta1, float beta2, float eps, float weight_decay,
                         int zero_sum);

/* The same update, which also measures the two vectors whose ratio is the gradient signal-to-noise ratio
 * of Section 5.2.1 (effect of batch size on DP gradients) while they pass through registers, at no extra
 * memory traffic:
 *     snr_sq[0] += sum_e sum[e]^2               (the aggregated clipped gradient, before the division by |B_t|)
 *     snr_sq[1] += sum_e (sigma*C*z_e)^2        (the noise vector added to it; 0 if sigma == 0)
 * over the slice's elements.  snr_sq is a DEVICE array of 2 floats that the caller clears (dp_zero_f32)
 * before the first slice of a step; squared norms add over slices, and the ratio is
 * sqrt(snr_sq[0] / snr_sq[1]).  Each workgroup reduces its elements in fp32 in a fixed order, the
 * per-workgroup pairs (library workspace: 8 bytes per 1024 elements; DP_ERR_WORKSPACE if that does not
 * fit) are added in fp64 in index order: results are reproducible run to run.  Everything else, argument
 * checks included, is dp_noise_adamw. */
dp_status dp_noise_adamw_snr(dp_ctx* ctx, float* params, float* m, float* v, float* sum, uint64_t n,
                             uint64_t elem_offset, float sigma, float C, uint64_t seed, uint64_t step,
                             uint64_t batch_size, float lr, float beta1, float beta2, float eps, float weight_decay,
                             int zero_sum, float* snr_sq);

/* dp_noise_adamw_snr for callers that cannot allocate device memory or hold a context whose creation does (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): no dp_ctx, the work is enqueued on
 * `hip_stream` (a hipStream_t, borrowed; NULL = the null stream), whose device must be the current device, and the
 * per-workgroup partial norms go to a fixed array in the library's device image (8 MiB per GPU, held until the process
 * ends; its address on a device is looked up by the first call on that device or by dp_create) instead of a workspace.
 * No hipMalloc / hipFree and no allocating library call.  Limit: n <= 2^30 elements per call, DP_ERR_WORKSPACE beyond
 * (slice the update: snr_sq adds over slices).  Same arguments, argument checks, kernels and results, bit for bit, as
 * dp_noise_adamw_snr; errors are returned as status codes only (there is no context to hold a message).  All calls on
 * one GPU share that GPU's array: every call overwrites the part it uses, nothing needs clearing, but calls that overlap in
 * time on one GPU (different streams or threads) race; calls on one stream are safe. */
dp_status dp_noise_adamw_snr_static(void* hip_stream, float* params, float* m, float* v, float* sum, uint64_t n,
                                    uint64_t elem_offset, float sigma, float C, uint64_t seed, uint64_t step,
                                    uint64_t batch_size, float lr, float beta1, float beta2, float eps, float weight_decay,
                                    int zero_sum, float* snr_sq);

/* ---------------------------------------------------------------------------------------------------
 * Aids
 * ------------------------------------------------------------------------------------------------- */
dp_status dp_zero_f32(dp_ctx* ctx, float* p, uint64_t n);
/* The raw Philox words that serve elements [elem_offset, elem_offset + n) (same mapping as above). */
dp_status dp_philox_u32(dp_ctx* ctx, uint32_t* out, uint64_t n, uint64_t elem_offset, uint64_t seed, uint64_t step);
/* The standard normals z that dp_noise_adamw draws for elements [elem_offset, elem_offset + n). */
dp_status dp_normal_f32(dp_ctx* ctx, float* out, uint64_t n, uint64_t elem_offset, uint64_t seed, uint64_t step);
/* Host-only, pure: the path DP_PATH_AUTO takes for this shape (HOST pointer out). */
dp_status dp_choose_path(int T, int d_in, int d_out, dp_dtype dtype, dp_path* out);
/* Host-only, pure: how the Gram path cuts the T x T plane of an example (128 < T <= 2048) into the units its workgroups
 * take.  The plane is nblk x nblk cells of 128 x 128, nblk = ceil(T / 128); only cells (r, c) with r <= c are formed.
 * Writes one word per unit to the HOST array `units` (capacity words) and their number to *n_units:
 *   bit 24 set:   a diagonal block of the panels a = bits 0-7 and b = bits 16-23: cells (a, a), (a, b), (b, b);
 *   bit 24 clear: a row pair, R = bits 0-7, C1 = bits 8-15, C2 = bits 16-23: cells (R, C1) and (R, C2), where (x, y) with
 *                 x > y stands for (y, x); C2 == 255: the cell (R, C1) alone.
 * DP_ERR_SHAPE if T is outside (128, 2048], DP_ERR_WORKSPACE if capacity is too small (70 words always suffice). */
dp_status dp_gram_unit_plan(int T, uint32_t* units, int capacity, int* n_units);


/* ---------------------------------------------------------------------------------------------------
 * Schedules: the per-step scalars q_t (batch size) and eta_t (learning rate) of Algorithm 1's input list.
 * Host-only, pure; `out` is a HOST pointer; `step` counts from 1; DP_ERR_VALUE on inconsistent arguments.
 *
 * dp_batch_size_schedule: the increasing batch-size schedule of Section 5.2.2 (batch size schedule improves efficiency): the
 * batch grows from b_start to b_end over ramp_steps steps in n_increments equal jumps of
 * floor((b_end - b_start) / n_increments), the k-th one once k/n_increments of the ramp's steps are complete,
 * the last one landing exactly on b_end (the paper's run: 262144 -> 1048576 over 7500 steps in 4 jumps of
 * 196608).  The caller turns q_t into a number of micro-batches and passes q_t as batch_size to the update.
 *
 * dp_lr_schedule: linear warm-up to `peak` at step == warmup_steps, then quadratic decay
 * peak * ((total_steps - step) / (total_steps - warmup_steps))^2, zero from total_steps on (the schedule named in
 * the hyper-parameter tuning section: 7500 warm-up steps of 20000; the exact form of the decay is not given there).
 * ------------------------------------------------------------------------------------------------- */
dp_status dp_batch_size_schedule(uint64_t step, uint64_t b_start, uint64_t b_end, uint64_t ramp_steps,
                                 uint32_t n_increments, uint64_t* out);
dp_status dp_lr_schedule(uint64_t step, double peak, uint64_t warmup_steps, uint64_t total_steps, double* out);

/* ---------------------------------------------------------------------------------------------------
 * Privacy accounting for a schedule of batch sizes (Section 3: Renyi-DP composition over steps with different
 * batch sizes, then translation to (eps, delta)).  Host-only, pure, double precision; out pointers are HOST
 * pointers.  Written from the cited papers (Mironov, "Renyi differential privacy"; Mironov, Talwar, Zhang,
 * "Renyi differential privacy of the sampled Gaussian mechanism"), integer orders only.
 *
 * dp_rdp_sampled_gaussian: eps(alpha) of ONE step that applies the Gaussian mechanism with noise multiplier sigma
 * to a Poisson sample of rate q = batch size / data-set size, for an integer order alpha >= 2:
 *     eps(alpha) = ln( sum_{k=0..alpha} C(alpha,k) (1-q)^(alpha-k) q^k exp((k^2-k) / (2 sigma^2)) ) / (alpha - 1).
 * dp_rdp_epsilon: a run of n_phases phases, phase p = steps[p] steps at rate q[p], is
 * (alpha, sum_p steps[p] * eps_p(alpha))-RDP; returns the smallest eps = RDP(alpha) + ln(1/delta) / (alpha - 1)
 * over alpha = 2 .. max_alpha and (if best_alpha is not NULL) the order that gives it.
 * dp_rdp_noise_multiplier: the noise multiplier of Algorithm 1 for a privacy target (Section 3: the accountant is what
 * gives sigma) - the smallest sigma, to a relative rel_tol in (0,1), for which dp_rdp_epsilon of the same run is at most
 * eps_target.  The guarantee decreases in sigma: the target is bracketed from sigma = 1 by doubling and halving and the
 * bracket bisected; the end that meets the target is returned in *sigma (a HOST pointer, like every pointer of these
 * three functions).  A run that needs no noise (no steps, q = 0) returns a value below 2^-9.  DP_ERR_VALUE if
 * eps_target <= 0 or no sigma up to 2^20 meets it (eps_target below ln(1/delta) / (max_alpha - 1)).
 * DP_ERR_VALUE for q outside [0,1], sigma <= 0, alpha < 2, delta outside (0,1).
 * ------------------------------------------------------------------------------------------------- */
dp_status dp_rdp_sampled_gaussian(double q, double sigma, int alpha, double* out);
dp_status dp_rdp_epsilon(const double* q, const uint64_t* steps, int n_phases, double sigma, double delta, int max_alpha,
                         double* eps, int* best_alpha);
dp_status dp_rdp_noise_multiplier(const double* q, const uint64_t* steps, int n_phases, double eps_target, double delta,
                                  int max_alpha, double rel_tol, double* sigma);

/* ---------------------------------------------------------------------------------------------------
 * Kernel timing (for benchmarks): while enabled, the library brackets each launch of its three main
 * kernels with HIP events on the context's stream.  dp_profile_read synchronises the stream and returns,
 * for one kernel kind, the summed launch duration in milliseconds, the launch count and the summed
 * algorithmic work (flops for DP_PROF_WGEMM: 2*B*T*d_in*d_out per launch; bytes for DP_PROF_GRAM:
 * B*T*(d_in+d_out)*elem, and for DP_PROF_ADAMW: 28 or 32 per element), then clears that kind's records.
 * All out pointers are HOST pointers and may be NULL.  At most 65536 launches are kept per enable.
 * ------------------------------------------------------------------------------------------------- */
typedef enum { DP_PROF_WGEMM = 0, DP_PROF_GRAM = 1, DP_PROF_ADAMW = 2 } dp_prof_kind;
dp_status dp_profile_enable(dp_ctx* ctx, int enable);
dp_status dp_profile_read(dp_ctx* ctx, dp_prof_kind kind, double* ms_total, uint64_t* launches, double* work_total);
/* Calibration for the roofline of the clip-weighted sum (the dominant kernel of Algorithm 1's g_t line): runs a loop of
 * nothing but the bf16 16x16x32 matrix instructions of that kernel (same accumulator tiles and waves per CU, operands
 * held in registers, pseudo-random values), `launches` launches of `iters` loop iterations each after one warm-up
 * launch, and returns the rate they sustain in TFLOP/s (*tflops, a HOST pointer): what the card's power limit leaves of
 * the nominal matrix peak.  Synchronises the stream.  iters in [1, 2^20], launches in [1, 1024], else DP_ERR_VALUE. */
dp_status dp_profile_mfma_ceiling(dp_ctx* ctx, int iters, int launches, double* tflops);

#ifdef __cplusplus
}
#endif
#endif /* DPCLIP_H */
