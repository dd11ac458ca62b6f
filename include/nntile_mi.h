/*
 * nntile_mi.h -- C ABI of the MI355X tile-operation library.
 *
 * The library carries out, on one gfx950 GPU, the tile-level tensor operations
 * that a task-based runtime dispatches when training a GPT-2 style transformer
 * (arxiv 2504.13236): a tensor is a shape plus a tile shape (section 2: data is
 * cut into tiles, operations into tasks that touch a few tiles; section 5: the
 * cut may run along every axis), each layer is a forward / backward pair of
 * operations on tiles (section 3), tasks are submitted one after another and run
 * asynchronously once the tiles they read are ready (section 2, sequential task
 * flow).
 *
 * General rules
 *  - Every call returns an int32 status: NNT_OK (0) or a negative error code.
 *    Nothing is thrown across this boundary.  nnt_last_error() gives the text of
 *    the last failure of a context (string owned by the context).
 *  - Pointers named `stream` are hipStream_t values passed as void* (NULL is the
 *    legacy default stream).  Pointers to tile data are DEVICE pointers; every
 *    other pointer (shapes, descriptors, out-parameters) is a HOST pointer.
 *  - The caller owns all tile memory.  On the device the library allocates only
 *    (a) descriptor tables: the tile-pointer table of every tensor, the tables of
 *    cached product plans and of grouped optimiser steps; (b) the fp32 scratch of
 *    the two-stage column sums (grows on demand, at least 4 MiB once used); (c)
 *    for products whose contraction is cut into k-slices, an fp32 workspace of
 *    slices x macro-tile partial sums per cached plan (at most 2 GiB each; a plan
 *    whose workspace would be larger is built without slices).  nnt_ctx_stats
 *    reports the bytes held for (a) and for (b) + (c).  Tables and workspaces of a
 *    plan are released when one of its tensors or the context is destroyed, the
 *    rest in the matching destroy call.
 *  - Element types: NNT_F32 (IEEE binary32) and NNT_BF16 (bfloat16, converted
 *    with round-to-nearest-even).  All arithmetic, reductions and accumulation
 *    are in fp32 whatever the storage type.
 *  - Layout: inside a tile the FIRST index runs fastest (column-major): element
 *    (i0, i1, i2, ...) of a tile with extents (n0, n1, n2, ...) sits at offset
 *    i0 + n0 * (i1 + n1 * (i2 + ...)).  Tiles of a tensor are separate buffers;
 *    the tile grid is enumerated first axis fastest as well.  A tile on the far
 *    edge of an axis is smaller when the base tile does not divide the extent.
 *  - A NULL tile pointer marks a tile of structural zeros: it is never read or
 *    written, contributes nothing to a product, and (for the attention scores)
 *    stands for a block that the causal mask removes entirely.
 *  - Tile-level calls (nnt_tile_*) only enqueue work on the given stream.
 *    Tensor-level calls (nnt_gemm, nnt_gelu, ...) submit tasks to the context's
 *    executor and return at once; results may be read after nnt_wait().
 *    Shape, type and tiling mismatches are reported synchronously by the call
 *    that submits; a device failure makes the context fail every later call with
 *    NNT_ESTATE until it is destroyed.
 *  - Not thread safe per context: one host thread submits (sequential task flow).
 */
#ifndef NNTILE_MI_H
#define NNTILE_MI_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* exported from the shared library; everything else in it is hidden */
#define NNT_API __attribute__((visibility("default")))

#define NNT_OK        0
#define NNT_EINVAL   (-1)   /* bad argument, shape or tiling mismatch            */
#define NNT_EDTYPE   (-2)   /* unsupported element type or type combination     */
#define NNT_EHIP     (-3)   /* HIP runtime call failed                          */
#define NNT_ENOMEM   (-4)   /* host or device allocation of a descriptor failed */
#define NNT_ESTATE   (-5)   /* context already failed, or call not allowed now  */

#define NNT_F32   0
#define NNT_BF16  1

#define NNT_OP_N  0         /* operand used as stored      */
#define NNT_OP_T  1         /* operand used transposed     */

#define NNT_GELU_TANH 0     /* 0.5 x (1 + tanh(sqrt(2/pi) (x + 0.044715 x^3))) */
#define NNT_GELU_ERF  1     /* 0.5 x (1 + erf(x / sqrt 2))                     */

#define NNT_GRAN_OP    0    /* one launch per tensor-level operation (a table of tile pointers) */
#define NNT_GRAN_TILE  1    /* one task and launch per tile (per output tile for products)      */

#define NNT_MAX_DIM 4

typedef struct nnt_ctx nnt_ctx;
typedef struct nnt_tensor nnt_tensor;
typedef struct nnt_gpt2_block nnt_gpt2_block;

/* ------------------------------------------------------------------------- */
/* Context and executor (section 2: task submission, sequential task flow).   */
/* ------------------------------------------------------------------------- */

/* Creates an executor on `device` with `n_streams` (1..8) HIP streams.  If
 * `caller_streams` is not NULL it holds n_streams hipStream_t values that the
 * context adopts (and never destroys); otherwise the context creates its own
 * non-blocking streams at default priority. */
NNT_API int32_t nnt_ctx_create(int32_t device, int32_t n_streams, void* const* caller_streams, nnt_ctx** out);
/* Waits for all submitted work, then frees the context's descriptors.  Tensors
 * and blocks created on it must be destroyed first. */
NNT_API int32_t nnt_ctx_destroy(nnt_ctx* ctx);
/* Blocks the host until every submitted task has finished. */
NNT_API int32_t nnt_wait(nnt_ctx* ctx);
/* Makes stream 0 wait (on the device, not the host) for everything submitted so
 * far on the other streams, so that an event recorded on stream 0 afterwards
 * covers all earlier tasks. */
NNT_API int32_t nnt_ctx_join(nnt_ctx* ctx);
/* hipStream_t number `i` of the context, as void*. */
NNT_API int32_t nnt_ctx_stream(nnt_ctx* ctx, int32_t i, void** out);
NNT_API const char* nnt_last_error(nnt_ctx* ctx);
/* serial != 0: every task goes to stream 0 in submission order (race checks). */
NNT_API int32_t nnt_ctx_set_serial(nnt_ctx* ctx, int32_t serial);
/* NNT_GRAN_OP (default) or NNT_GRAN_TILE. */
NNT_API int32_t nnt_ctx_set_granularity(nnt_ctx* ctx, int32_t granularity);

typedef struct nnt_exec_stats {
    int64_t tasks;          /* tasks submitted since creation                       */
    int64_t launches;       /* kernel launches issued                               */
    int64_t event_waits;    /* cross-stream dependencies turned into event waits    */
    int64_t plans;          /* product plans (descriptor tables) built and cached   */
    int64_t device_table_bytes;      /* device memory held for descriptor tables             */
    int64_t device_workspace_bytes;  /* device memory held for reduction scratch and the
                                        k-slice workspaces of the cached product plans       */
} nnt_exec_stats;
NNT_API int32_t nnt_ctx_stats(nnt_ctx* ctx, nnt_exec_stats* out);

/* Per-task timing for measurements.  While enabled, every task is bracketed by a
 * pair of timing events on the stream it runs on; nnt_profile_read waits for all
 * work and returns one entry per operation label (at most `capacity` entries are
 * written, *n_out is the number that exist): tasks, kernel launches, summed
 * device time, and the algorithmic work the operations stand for (flops for
 * products, bytes for memory-bound operations: the bytes that one pass over the
 * operands moves).  Enabling clears earlier records.  Not available during capture. */
typedef struct nnt_profile_entry {
    char    label[112];
    int64_t tasks;
    int64_t launches;
    double  ms;
    double  work;
    int32_t work_is_bytes;
    int32_t reserved;
} nnt_profile_entry;
NNT_API int32_t nnt_profile_enable(nnt_ctx* ctx, int32_t on);
NNT_API int32_t nnt_profile_read(nnt_ctx* ctx, nnt_profile_entry* out, int32_t capacity, int32_t* n_out);

/* Host-only replay of the executor's decisions (section 2, task submission: tasks are
 * submitted in sequence and run asynchronously, ordered only by their data): for
 * n_tasks tasks over n_tiles tiles -- task t accesses the tiles
 * acc_tile[task_first[t] .. task_first[t+1]-1] with the modes acc_mode[...]
 * (1 read, 2 write, 3 read-write, 6 + 256 * p write of part p of the tile: writers of
 * different parts of a tile are not ordered among themselves, as the attention products
 * that write the rows of Q, K and V inside one tensor) -- reports the stream each task would run on, its
 * sequence number on that stream, and per task NNT_MAX_STREAMS entries: the sequence
 * number on every other stream that it would wait for (0 = none).  Uses the same
 * code as the executor, touches no device: it lets a test check on the CPU that
 * every read-after-write, write-after-read and write-after-write pair is ordered.
 * All pointers are host memory. */
#define NNT_MAX_STREAMS 8
NNT_API int32_t nnt_sched_simulate(int32_t n_streams, int32_t serial, int32_t n_tiles, int32_t n_tasks,
                           const int32_t* task_first, const int32_t* acc_tile, const int32_t* acc_mode,
                           int32_t* stream_out, int64_t* seq_out, int64_t* wait_seq_out);

/* Stream capture of the task flow into a HIP graph (section 2: the graph of a
 * training iteration repeats, so it can be built once and replayed).  Between
 * begin and end, tensor-level calls are recorded instead of run; every plan they
 * need must already exist (run the same calls once before capturing).  Captured
 * tasks are spread over at most two streams.  The graph replays on stream 0. */
typedef struct nnt_graph nnt_graph;
NNT_API int32_t nnt_capture_begin(nnt_ctx* ctx);
NNT_API int32_t nnt_capture_end(nnt_ctx* ctx, nnt_graph** out);
NNT_API int32_t nnt_graph_launch(nnt_graph* g);
NNT_API int32_t nnt_graph_destroy(nnt_graph* g);

/* ------------------------------------------------------------------------- */
/* Tiled tensors (section 2: tiles; section 5: split along all axes).          */
/* ------------------------------------------------------------------------- */

/* Number of tiles of a tensor with `shape` cut by `basetile` (1..4 axes). */
NNT_API int32_t nnt_tiling_ntiles(int32_t ndim, const int64_t* shape, const int64_t* basetile, int64_t* out);
/* Extents of tile number `tile_index` (grid order, first axis fastest). */
NNT_API int32_t nnt_tiling_tile_shape(int32_t ndim, const int64_t* shape, const int64_t* basetile,
                              int64_t tile_index, int64_t* shape_out);

/* Describes a tensor: the call copies shape, base tile and the `ntiles` device
 * pointers (grid order); it allocates no tile memory and never frees any. */
NNT_API int32_t nnt_tensor_create(nnt_ctx* ctx, int32_t dtype, int32_t ndim, const int64_t* shape,
                          const int64_t* basetile, void* const* tile_ptrs, nnt_tensor** out);
/* Waits for tasks that still use the tensor, then frees its descriptors. */
NNT_API int32_t nnt_tensor_destroy(nnt_tensor* t);
NNT_API int32_t nnt_tensor_ntiles(const nnt_tensor* t, int64_t* out);
NNT_API int32_t nnt_tensor_tile_shape(const nnt_tensor* t, int64_t tile_index, int64_t* shape_out);
NNT_API int32_t nnt_tensor_tile_bytes(const nnt_tensor* t, int64_t tile_index, int64_t* out);

/* ------------------------------------------------------------------------- */
/* Single-tile kernels.  n, m, ... count elements; all buffers are contiguous   */
/* tiles in the layout above unless a leading dimension is given.               */
/* ------------------------------------------------------------------------- */

/* C = alpha * op(A) * op(B) + beta * C for `batch` independent matrices (section
 * 3, linear and attention layers: products and sums of elementary tiles).
 * op(A) is m x k, op(B) is k x n, C is m x n, all column-major with leading
 * dimensions lda/ldb/ldc (in elements) and a stride (in elements) between
 * consecutive batch members.  A and B have type dtype_in, C dtype_out; products
 * are accumulated in fp32 and rounded once.  beta == 0 never reads C. */
NNT_API int32_t nnt_tile_gemm(void* stream, int32_t dtype_in, int32_t dtype_out, int32_t opA, int32_t opB,
                      int64_t m, int64_t n, int64_t k, int64_t batch, float alpha,
                      const void* A, int64_t lda, int64_t strideA,
                      const void* B, int64_t ldb, int64_t strideB,
                      float beta, void* C, int64_t ldc, int64_t strideC);

/* x[0..n) = value. */
NNT_API int32_t nnt_tile_fill(void* stream, int32_t dtype, int64_t n, float value, void* x);
/* y = alpha * x + beta * y (residual add and gradient fan-in). */
NNT_API int32_t nnt_tile_add(void* stream, int32_t dtype, int64_t n, float alpha, const void* x, float beta, void* y);
/* y[i] = x[i] converted from dtype_in to dtype_out. */
NNT_API int32_t nnt_tile_cast(void* stream, int32_t dtype_in, int32_t dtype_out, int64_t n, const void* x, void* y);
/* Copies an up-to-4-axis block between two tiles: element (i0..i3) of the block
 * is read at src + sum i_a * src_stride[a] and written at dst + sum i_a *
 * dst_stride[a] (strides in elements).  The head split / merge of the attention
 * layer is made of such copies. */
NNT_API int32_t nnt_tile_copy_block(void* stream, int32_t dtype, int32_t ndim, const int64_t* extent,
                            const void* src, const int64_t* src_stride,
                            void* dst, const int64_t* dst_stride);

/* Y (m x n, m fastest) += bias (fp32, length m), the same bias in every column
 * (section 3, linear layer: the "+." of Y = W X +. b). */
NNT_API int32_t nnt_tile_bias_add(void* stream, int32_t dtype, int64_t m, int64_t n, const float* bias, void* Y);
/* db (fp32, length m) = sum over the n columns of dY, added to the old db when
 * accumulate != 0 (gradient of the bias).  `scratch` is fp32 device memory of at
 * least nnt_tile_bias_grad_scratch(m, n) elements. */
NNT_API int64_t nnt_tile_bias_grad_scratch(int64_t m, int64_t n);
NNT_API int32_t nnt_tile_bias_grad(void* stream, int32_t dtype, int64_t m, int64_t n, const void* dY,
                           float* db, int32_t accumulate, float* scratch);

/* nnt_tile_bias_grad for callers that cannot allocate (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same kernels
 * and result, but the partial column sums go to a static device array inside
 * the library (4 MiB per GPU, held until the process ends) instead of caller
 * scratch.  Neither allocates nor frees anything.  Limit: nnt_tile_bias_grad_scratch(m, n)
 * <= nnt_tile_bias_grad_static_max() (2^20 fp32 elements), else NNT_EINVAL and
 * nothing is launched.  The array's device address is looked up once per GPU:
 * by nnt_ctx_create on that GPU, else by the first call (make that first call
 * outside a capture).  All calls on one GPU share the array: calls that may
 * overlap (different streams without an ordering between them) race; calls on
 * one stream, or ordered by events, are safe.  dY, db are device pointers the
 * caller owns; the call is asynchronous on `stream`. */
NNT_API int64_t nnt_tile_bias_grad_static_max(void);
NNT_API int32_t nnt_tile_bias_grad_static(void* stream, int32_t dtype, int64_t m, int64_t n, const void* dY,
                                  float* db, int32_t accumulate);

/* y = gelu(x); dx = dy * gelu'(x)  (section 3, nonlinear activations). */
NNT_API int32_t nnt_tile_gelu(void* stream, int32_t dtype, int32_t variant, int64_t n, const void* x, void* y);
NNT_API int32_t nnt_tile_gelu_bwd(void* stream, int32_t dtype, int32_t variant, int64_t n,
                          const void* x, const void* dy, void* dx);

/* Layer normalisation over the first axis, in the paper's tile steps (section 3,
 * layer normalization).  x is an m x n tile: m features of n tokens, one of the
 * tiles along the embedding axis.  stats is fp32 [2][n].
 *  step 1  nnt_tile_ln_stats: folds this tile's per-token mean and sum of
 *          squared deviations into stats, which already covers `count_before`
 *          features (0 for the first tile).  When finalize_total > 0 it must
 *          equal count_before + m and stats becomes (mean, 1/sqrt(var + eps))
 *          with the biased variance.
 *  steps 2 and 3  nnt_tile_ln_apply: y = gamma * (x - mean) * rstd + beta, with
 *          gamma and beta the fp32 slices (length m) that belong to this tile. */
NNT_API int32_t nnt_tile_ln_stats(void* stream, int32_t dtype, int64_t m, int64_t n, const void* x,
                          float* stats, int64_t count_before, int64_t finalize_total, float eps);
NNT_API int32_t nnt_tile_ln_apply(void* stream, int32_t dtype, int64_t m, int64_t n, const void* x,
                          const float* stats, const float* gamma, const float* beta, void* y);
/* Backward.  sums is fp32 [2][n]: per-token sums over the features of g = dy *
 * gamma and of g * xhat; `init` != 0 overwrites instead of adding.
 * nnt_tile_ln_bwd_dx: dx = rstd * (g - sums0 / N_e - xhat * sums1 / N_e)
 * (+ dres when dres is not NULL: the gradient that arrives over the residual
 * connection). */
NNT_API int32_t nnt_tile_ln_bwd_sums(void* stream, int32_t dtype, int64_t m, int64_t n, const void* x,
                             const float* stats, const float* gamma, const void* dy,
                             float* sums, int32_t init);
NNT_API int32_t nnt_tile_ln_bwd_dx(void* stream, int32_t dtype, int64_t m, int64_t n, int64_t N_e,
                           const void* x, const float* stats, const float* gamma, const void* dy,
                           const float* sums, const void* dres, void* dx);
/* dgamma, dbeta (fp32, length m) = sum over the n tokens of dy * xhat and of dy;
 * added to the old values when accumulate != 0.  scratch: fp32, at least
 * nnt_tile_ln_bwd_params_scratch(m, n) elements. */
NNT_API int64_t nnt_tile_ln_bwd_params_scratch(int64_t m, int64_t n);
NNT_API int32_t nnt_tile_ln_bwd_params(void* stream, int32_t dtype, int64_t m, int64_t n, const void* x,
                               const float* stats, const void* dy, float* dgamma, float* dbeta,
                               int32_t accumulate, float* scratch);

/* Softmax over the first axis in the paper's two subroutines (section 3,
 * SoftMax).  a is a tile of tk x tq x batch scores (tk keys fastest); stats is
 * fp32 [2][tq][batch] = (running maximum, running sum of exp(t - maximum)).
 * (k0, q0) is the position of the tile's first key and query in the whole
 * sequence; with causal != 0 a score whose key index exceeds its query index is
 * excluded.  Scores are multiplied by `scale` before use.
 *  subroutine 1  nnt_tile_softmax_stats: folds this tile's maximum and
 *                denominator into stats (`init` != 0: stats start empty).
 *  subroutine 2  nnt_tile_softmax_apply: a = exp(scale * a - max) / sum, in place
 *                (0 for excluded scores). */
NNT_API int32_t nnt_tile_softmax_stats(void* stream, int32_t dtype, int64_t tk, int64_t tq, int64_t batch,
                               int64_t k0, int64_t q0, int32_t causal, float scale,
                               const void* a, float* stats, int32_t init);
NNT_API int32_t nnt_tile_softmax_apply(void* stream, int32_t dtype, int64_t tk, int64_t tq, int64_t batch,
                               int64_t k0, int64_t q0, int32_t causal, float scale,
                               void* a, const float* stats);
/* Backward: dots (fp32 [tq][batch]) (+)= sum_k p * dp;  dp = p * (dp - dots) in place. */
NNT_API int32_t nnt_tile_softmax_bwd_dot(void* stream, int32_t dtype, int64_t tk, int64_t tq, int64_t batch,
                                 const void* p, const void* dp, float* dots, int32_t init);
NNT_API int32_t nnt_tile_softmax_bwd_apply(void* stream, int32_t dtype, int64_t tk, int64_t tq, int64_t batch,
                                   const void* p, void* dp, const float* dots);

/* One Adam step number `step` (>= 1) on n parameters (section 3, optimizers;
 * Kingma & Ba with bias correction, eps outside the square root; weight_decay
 * > 0 gives the decoupled AdamW form).  g, p, m, v are fp32; p_lowp, when not
 * NULL, receives the bf16 copy of the updated parameters. */
NNT_API int32_t nnt_tile_adam(void* stream, int64_t n, int32_t step, double lr, double beta1, double beta2,
                      double eps, double weight_decay, const float* g, float* p, float* m, float* v,
                      void* p_lowp);
/* One tile of the SGD-with-momentum step (formulas at nnt_sgd_step); n fp32
 * elements of g, p, v; p_lowp: bf16 copy of the new p, or NULL. */
NNT_API int32_t nnt_tile_sgd(void* stream, int64_t n, double lr, double momentum, double weight_decay,
                     int32_t nesterov, const float* g, float* p, float* v, void* p_lowp);

/* ------------------------------------------------------------------------- */
/* Tensor-level operations: walk the tile grid and submit tasks.               */
/* ------------------------------------------------------------------------- */

/* C = alpha * op(A) . op(B) + beta * C on tiled tensors.  The last n_batch_axes
 * axes of A, B and C are batch axes (equal extents and tiling).  Of the other
 * axes, the n_contract_axes contracted ones are A's last (opA = N) or first
 * (opA = T) and B's first (opB = N) or last (opB = T); C's axes are A's free
 * axes, B's free axes, then the batch axes.  Inside a tile each axis group
 * flattens to a column-major matrix.  Contracted axes, and free axes against
 * C's, must be tiled alike.  For every C tile the products over the contracted
 * tiles are summed in fp32 registers and rounded once.  `bias` (fp32 tensor of
 * one axis tiled like C's first axis, or NULL) is added to every column. */
NNT_API int32_t nnt_gemm(nnt_ctx* ctx, float alpha, int32_t opA, nnt_tensor* A, int32_t opB, nnt_tensor* B,
                 float beta, nnt_tensor* C, int32_t n_contract_axes, int32_t n_batch_axes,
                 nnt_tensor* bias);
/* The same product with the beta term taken from a second tensor: C = alpha * op(A) * op(B) +.
 * bias + beta * R (section 3: a linear layer whose result is added to the layer's input, as
 * the residual connections of a transformer block do), in one pass over C.  R has C's type,
 * shape and tiling and a tile wherever C has one; it is only read.  R = NULL or R = C is
 * nnt_gemm. */
NNT_API int32_t nnt_gemm_res(nnt_ctx* ctx, float alpha, int32_t opA, nnt_tensor* A, int32_t opB, nnt_tensor* B,
                     float beta, nnt_tensor* C, int32_t n_contract_axes, int32_t n_batch_axes, nnt_tensor* bias,
                     nnt_tensor* R);
/* A linear layer with the activation that follows it (section 3: the MLP is linear, GELU, linear):
 * C = alpha * op(A) . op(B) +. bias and G = gelu(C) leave one launch, so the activation is not a pass
 * of its own over C.  No batch axes; G has C's type, shape and tiling, a tile wherever C has one, and
 * is neither A, B nor C; it is written, C too (both are kept: the backward pass needs C).  One launch
 * for fp32 tensors whose tiles are whole macro-tiles of the direct-load kernels with op(B) = B; any
 * other form runs nnt_gemm and nnt_gelu one after the other (same result).  variant: NNT_GELU_*. */
NNT_API int32_t nnt_gemm_gelu(nnt_ctx* ctx, float alpha, int32_t opA, nnt_tensor* A, int32_t opB, nnt_tensor* B,
                      nnt_tensor* C, int32_t n_contract_axes, nnt_tensor* bias, int32_t variant, nnt_tensor* G);
/* The adjoint of that pair, seen from the next layer: C = (alpha * op(A) . op(B)) * gelu'(X) element by
 * element (section 3: the gradient that the second linear layer sends back, times the activation's
 * derivative at the first layer's result X).  X is only read; same conditions on it as on G above
 * (one launch: fp32, whole macro-tiles, op(A) = A^T, op(B) = B; else nnt_gemm, then nnt_gelu_bwd). */
NNT_API int32_t nnt_gemm_gelu_bwd(nnt_ctx* ctx, float alpha, int32_t opA, nnt_tensor* A, int32_t opB, nnt_tensor* B,
                          nnt_tensor* C, int32_t n_contract_axes, int32_t variant, nnt_tensor* X);

/* The per-head products of the attention layer (section 3, attention layer: K^T Q, V P and their four
 * adjoint products, one per batch member and head) on tensors that keep the heads side by side along their
 * first axis, as the linear layers around the attention produce and consume them, so that no copy into a
 * per-head layout is needed.  C = alpha * op(A) . op(B), one contracted axis, batch axes (N_b, N_h).
 * Each of A, B, C is given with a part number:
 *   part >= 0: a tensor [n_parts * N_h * h, N_s, N_b]; its rows [part * N_h * h, (part + 1) * N_h * h) are
 *              taken as [h, N_s, N_b, N_h] (row head * h + d is component d of that head).  Its row tiles
 *              must hold whole heads (base % h == 0) and a part whole row tiles (N_h * h % base == 0), and all
 *              its tiles must be present.  As C, only the rows of the part are written.
 *   part < 0:  a tensor [., ., N_b, N_h] as nnt_gemm(n_contract_axes = 1, n_batch_axes = 2) takes it (the
 *              scores and their adjoint); its head axis must be tiled in multiples of base / h heads.
 * At least one part must be >= 0, and the tensors with parts share one row tiling.  Host pointers to
 * descriptors; data stays where the tensors' tiles are.  The product is one launch whatever the context's
 * granularity; its tasks are ordered by whole tensors.  Errors: NNT_EINVAL for geometry that does not fit. */
NNT_API int32_t nnt_gemm_heads(nnt_ctx* ctx, float alpha, int32_t opA, nnt_tensor* A, int32_t partA, int32_t opB, nnt_tensor* B,
                       int32_t partB, nnt_tensor* C, int32_t partC, int32_t h, int32_t N_h);

NNT_API int32_t nnt_fill(nnt_ctx* ctx, float value, nnt_tensor* X);
NNT_API int32_t nnt_add(nnt_ctx* ctx, float alpha, nnt_tensor* X, float beta, nnt_tensor* Y);
NNT_API int32_t nnt_cast(nnt_ctx* ctx, nnt_tensor* X, nnt_tensor* Y);
/* Y[d, ...] += b[d]; db[d] = sum over the other axes of dY[d, ...]. */
NNT_API int32_t nnt_bias_add(nnt_ctx* ctx, nnt_tensor* b, nnt_tensor* Y);
NNT_API int32_t nnt_bias_grad(nnt_ctx* ctx, nnt_tensor* dY, nnt_tensor* db);
NNT_API int32_t nnt_gelu(nnt_ctx* ctx, int32_t variant, nnt_tensor* X, nnt_tensor* Y);
NNT_API int32_t nnt_gelu_bwd(nnt_ctx* ctx, int32_t variant, nnt_tensor* X, nnt_tensor* dY, nnt_tensor* dX);
/* X, Y: [N_e, N_s, N_b]; gamma, beta: fp32 [N_e] tiled like X's first axis;
 * stats: fp32 [2, N_s, N_b] tiled like X's other axes. */
NNT_API int32_t nnt_layernorm_fwd(nnt_ctx* ctx, nnt_tensor* X, nnt_tensor* gamma, nnt_tensor* beta, float eps,
                          nnt_tensor* Y, nnt_tensor* stats);
/* dX = layer-norm adjoint (+ dRes when not NULL); dgamma, dbeta overwritten. */
NNT_API int32_t nnt_layernorm_bwd(nnt_ctx* ctx, nnt_tensor* X, nnt_tensor* stats, nnt_tensor* gamma,
                          nnt_tensor* dY, nnt_tensor* dRes, nnt_tensor* dX,
                          nnt_tensor* dgamma, nnt_tensor* dbeta);
/* A: scores [N_k, N_q, batch axes...], softmax over the first axis, in place;
 * stats: fp32 [2, N_q, ...] tiled like A's other axes. */
NNT_API int32_t nnt_softmax_fwd(nnt_ctx* ctx, nnt_tensor* A, nnt_tensor* stats, float scale, int32_t causal);
/* dP <- P o (dP - sum_k P o dP), in place on dP. */
NNT_API int32_t nnt_softmax_bwd(nnt_ctx* ctx, nnt_tensor* P, nnt_tensor* dP);
/* Z: [n_parts * N_h * h, N_s, N_b]  <->  parts[p]: [h, N_s, N_b, N_h]; row
 * (p * N_h + j) * h + i of Z is component i of head j of part p (section 3,
 * attention layer: Q, K, V of size h x N_s x N_b x N_h). */
NNT_API int32_t nnt_head_split(nnt_ctx* ctx, nnt_tensor* Z, int32_t n_parts, nnt_tensor* const* parts);
NNT_API int32_t nnt_head_merge(nnt_ctx* ctx, int32_t n_parts, nnt_tensor* const* parts, nnt_tensor* Z);

/* Fused tile attention (section 3, attention layer and SoftMax): what the three
 * operations "scores, softmax over the keys, product with the values" compute,
 * in one kernel that walks the key tiles of each query tile and carries the
 * SoftMax subroutines' running column statistics (maximum, sum of shifted
 * exponentials) along instead of storing the N_s x N_s scores:
 *   B[i,q,b,j] = sum_k V[i,k,b,j] P[k,q,b,j],
 *   P[.,q,b,j] = softmax over k of scale * sum_i K[i,k,b,j] Q[i,q,b,j],
 * with causal != 0 over the keys k <= q only; scale > 0.  Q, K, V, B: [h, N_s, N_b, N_h]
 * tensors of one dtype (fp32 or bf16), tiled alike, first axis untiled, h = 64 or
 * 128, every tile present and 16-byte aligned; stats: fp32 [2, N_s, N_b, N_h]
 * tiled like their other axes, overwritten with the final (maximum of the scaled
 * scores, sum of exp(score - maximum)) of every column.  One task for the whole
 * tensor, or one per query tile at tile granularity.  At most 65535 blocks of
 * 128 queries (counted per sequence tile).
 * Errors: NNT_EINVAL (shape, tiling, missing tile), NNT_EDTYPE. */
NNT_API int32_t nnt_attention_fwd(nnt_ctx* ctx, nnt_tensor* Q, nnt_tensor* K, nnt_tensor* V, float scale,
                          int32_t causal, nnt_tensor* B, nnt_tensor* stats);
/* Its adjoint, recomputing the probabilities from Q, K and the statistics that
 * the forward call left: with D[q] = sum_i dB[i,q] B[i,q] and
 * dA[k,q] = P[k,q] (sum_i V[i,k] dB[i,q] - D[q]),
 *   dV[i,k] = sum_q dB[i,q] P[k,q],  dQ[i,q] = scale sum_k K[i,k] dA[k,q],
 *   dK[i,k] = scale sum_q Q[i,q] dA[k,q]        (per batch element and head).
 * B, stats: the forward call's outputs; dQ, dK, dV (tiled like Q) are overwritten.
 * One task of two kernels (dQ, then dK and dV); uses the context's reduction
 * scratch (2 N_s N_b N_h floats), which must exist before a graph capture. */
NNT_API int32_t nnt_attention_bwd(nnt_ctx* ctx, nnt_tensor* Q, nnt_tensor* K, nnt_tensor* V, nnt_tensor* B,
                          nnt_tensor* stats, nnt_tensor* dB, float scale, int32_t causal,
                          nnt_tensor* dQ, nnt_tensor* dK, nnt_tensor* dV);
/* The same two operations on tensors that keep the heads side by side along their first axis
 * (section 3, attention layer: what the linear layers before and after it produce and consume), so
 * that no per-head copies are needed: QKV and dQKV are [3 * N_h * h, N_s, N_b] with Q, K, V (their
 * adjoints) in rows [0, N_h h), [N_h h, 2 N_h h), [2 N_h h, 3 N_h h); Bm and dBm are [N_h * h, N_s, N_b];
 * row head * h + d is component d of that head.  All share one tiling whose row tiles hold whole heads
 * and divide N_h * h; h is 64 or 128; stats is fp32 (2, N_s, N_b, N_h) tiled like them along N_s and N_b.
 * One launch (two for the adjoint) whatever the context's granularity.  Errors as above. */
NNT_API int32_t nnt_attention_fwd_heads(nnt_ctx* ctx, nnt_tensor* QKV, float scale, int32_t causal, nnt_tensor* Bm,
                                nnt_tensor* stats, int32_t N_h);
NNT_API int32_t nnt_attention_bwd_heads(nnt_ctx* ctx, nnt_tensor* QKV, nnt_tensor* Bm, nnt_tensor* stats, nnt_tensor* dBm,
                                float scale, int32_t causal, nnt_tensor* dQKV, int32_t N_h);

typedef struct nnt_adam_cfg {
    double lr, beta1, beta2, eps, weight_decay;   /* doubles: 1 - beta is formed before rounding to fp32 */
} nnt_adam_cfg;
/* G, P, M, V: fp32 tensors tiled alike; P_lowp: bf16 tensor tiled alike or NULL. */
NNT_API int32_t nnt_adam_step(nnt_ctx* ctx, const nnt_adam_cfg* cfg, int32_t step, nnt_tensor* G, nnt_tensor* P,
                      nnt_tensor* M, nnt_tensor* V, nnt_tensor* P_lowp);

/* Embedding layer (section 3, Embedding layer): every token of the N_s x N_b
 * input gets its embedding vector, Y[e, s, b] = W[e, tokens[s + N_s * b]].
 * tokens: device pointer to N_s * N_b int32 (not tiled); W: [N_e, N_v] (one column
 * per vocabulary item), Y: [N_e, N_s, N_b], fp32 or bf16 each, any tiling.  A
 * token outside [0, N_v) yields a zero vector. */
NNT_API int32_t nnt_embedding_fwd(nnt_ctx* ctx, const int32_t* tokens, nnt_tensor* W, nnt_tensor* Y);
/* Its adjoint: dW[e, v] += sum of dY[e, s, b] over the positions whose token is v
 * (dW: fp32, accumulated into: clear it first; out-of-range tokens add nothing).
 * Positions that share a token are summed with floating-point atomics, so the
 * summation order, and with it the last bits, can differ from run to run. */
NNT_API int32_t nnt_embedding_bwd(nnt_ctx* ctx, const int32_t* tokens, nnt_tensor* dY, nnt_tensor* dW);
/* Cross-entropy loss (section 3, Cross-Entropy loss) over logits split into tiles,
 * L = - sum_{s,b} log(exp(x[c,s,b]) / sum_j exp(x[j,s,b])), c = labels[s + N_s * b]:
 * the SoftMax subroutines give the running (maximum, sum of shifted exponentials)
 * per column (stats, fp32 [2, N_s, N_b] tiled like X's other axes) and the
 * probabilities in place; then the label's entry of every column gives that
 * column's loss and is decreased by one, which leaves dL/dx in X.
 * X: [N_v, N_s, N_b] logits, fp32 or bf16, overwritten with the gradient;
 * labels: device pointer to N_s * N_b int32 in [0, N_v) (a label outside adds no
 * loss and leaves its column's probabilities); losses: device buffer of
 * N_s * N_b floats (per-column losses); loss: device float, their sum (summed
 * in a fixed order).  The caller owns both and must not reuse them before
 * nnt_wait or a later operation on X. */
NNT_API int32_t nnt_cross_entropy(nnt_ctx* ctx, nnt_tensor* X, const int32_t* labels, nnt_tensor* stats,
                          float* losses, float* loss);

/* SGD with momentum (section 3, Optimizers: the update is a weighted sum of the
 * parameter, the gradient and the momentum term):
 *   g' = g + weight_decay * p;  v <- momentum * v + g';
 *   p <- p - lr * v            (nesterov != 0:  p <- p - lr * (g' + momentum * v)).
 * With v = 0 before the first step this is the usual first step v = g'.
 * G, P, V: fp32 tensors tiled alike; P_lowp: bf16 tensor tiled alike or NULL. */
typedef struct nnt_sgd_cfg {
    double lr, momentum, weight_decay;
    int32_t nesterov;
} nnt_sgd_cfg;
NNT_API int32_t nnt_sgd_step(nnt_ctx* ctx, const nnt_sgd_cfg* cfg, nnt_tensor* G, nnt_tensor* P, nnt_tensor* V,
                     nnt_tensor* P_lowp);

/* ------------------------------------------------------------------------- */
/* One GPT-2 block (pre-LN, biases on all four linear layers, causal attention, */
/* no dropout): forward, backward and Adam as a flow of the tasks above.        */
/* ------------------------------------------------------------------------- */

typedef struct nnt_gpt2_block_cfg {
    int64_t N_e, N_h, N_m, N_s, N_b;    /* embedding, heads, MLP width, sequence, batch */
    int64_t tile_e, tile_m, tile_s;     /* base tiles on embedding-like, MLP and sequence axes */
    int64_t tile_b, tile_j, tile_i;     /* base tiles on batch, head-count and head-size axes   */
    int32_t dtype;                      /* NNT_F32 or NNT_BF16 storage of activations           */
    int32_t gelu_variant;
    float   eps;                        /* layer-norm epsilon (inside the square root)          */
    int32_t causal;
    int32_t fused_attention;            /* 0: scores, softmax and the product with V as three operations on a stored
                                           N_s x N_s tensor (the paper's flow); 1: nnt_attention_fwd / _bwd, which
                                           needs tile_i >= N_e / N_h; the slots P and DP are then unused */
} nnt_gpt2_block_cfg;

/* Tensors of a block.  The caller asks nnt_gpt2_block_slot() for the type, shape
 * and tiling of each slot, allocates its tiles, creates the nnt_tensor and hands
 * all of them over in one array indexed by slot. */
enum {
    /* parameters, fp32 */
    NNT_BLK_W_QKV = 0, NNT_BLK_W_O, NNT_BLK_W_1, NNT_BLK_W_2,
    NNT_BLK_B_QKV, NNT_BLK_B_O, NNT_BLK_B_1, NNT_BLK_B_2,
    NNT_BLK_GAMMA1, NNT_BLK_BETA1, NNT_BLK_GAMMA2, NNT_BLK_BETA2,
    /* parameter gradients, fp32 (same order: NNT_BLK_GRAD + parameter slot) */
    NNT_BLK_GRAD = 12,
    /* Adam moments, fp32 (NNT_BLK_ADAM_M + parameter slot, NNT_BLK_ADAM_V + ...); optional */
    NNT_BLK_ADAM_M = 24, NNT_BLK_ADAM_V = 36,
    /* bf16 copies of the four weight matrices (bf16 blocks only) */
    NNT_BLK_LOWP = 48,
    /* saved activations */
    NNT_BLK_STATS1 = 52, NNT_BLK_X1, NNT_BLK_QKV, NNT_BLK_Q, NNT_BLK_K, NNT_BLK_V,
    NNT_BLK_P, NNT_BLK_SM_STATS, NNT_BLK_BH, NNT_BLK_BM, NNT_BLK_X2, NNT_BLK_STATS2,
    NNT_BLK_X3, NNT_BLK_H1, NNT_BLK_G,
    /* backward work tensors */
    NNT_BLK_DG, NNT_BLK_DX3, NNT_BLK_DX2, NNT_BLK_DBM, NNT_BLK_DBH, NNT_BLK_DP,
    NNT_BLK_DQ, NNT_BLK_DK, NNT_BLK_DV, NNT_BLK_DQKV, NNT_BLK_DX1,
    NNT_BLK_NSLOTS
};

typedef struct nnt_slot_info {
    int32_t used;                 /* 0: this configuration has no such tensor              */
    int32_t dtype;
    int32_t ndim;
    int32_t causal_tiles;         /* 1: tiles (kt, qt, ...) with kt > qt are structural zeros (NULL) */
    int64_t shape[NNT_MAX_DIM];
    int64_t basetile[NNT_MAX_DIM];
} nnt_slot_info;

NNT_API int32_t nnt_gpt2_block_slot(const nnt_gpt2_block_cfg* cfg, int32_t slot, nnt_slot_info* out);
/* `slots` has NNT_BLK_NSLOTS entries; unused or optional ones (Adam moments) may
 * be NULL.  The block keeps the pointers, not the tensors' ownership. */
NNT_API int32_t nnt_gpt2_block_create(nnt_ctx* ctx, const nnt_gpt2_block_cfg* cfg, nnt_tensor* const* slots,
                              nnt_gpt2_block** out);
NNT_API int32_t nnt_gpt2_block_destroy(nnt_gpt2_block* blk);
/* X, Out, dOut, dX: [N_e, N_s, N_b] tensors of the block's dtype, tiled (tile_e,
 * tile_s, tile_b).  forward keeps X (by reference) for backward.  Where the row tiles
 * hold whole heads and divide N_e (whole-operation launches) the attention works on
 * NNT_BLK_QKV, NNT_BLK_BM, NNT_BLK_DBM and NNT_BLK_DQKV directly (nnt_gemm_heads, or
 * nnt_attention_fwd_heads / _bwd_heads with fused attention) and the per-head slots Q, K, V,
 * BH, DBH, DQ, DK, DV stay untouched; otherwise those are filled by head split / merge passes. */
NNT_API int32_t nnt_gpt2_block_forward(nnt_gpt2_block* blk, nnt_tensor* X, nnt_tensor* Out);
NNT_API int32_t nnt_gpt2_block_backward(nnt_gpt2_block* blk, nnt_tensor* dOut, nnt_tensor* dX);
/* Adam step on all 12 parameters; bf16 blocks also refresh the bf16 weight copies.
 * With one launch per operation the twelve tensors are updated by a single launch;
 * the first such call allocates two small device tables (tile pointers, tile sizes),
 * so it must come before nnt_capture_begin (NNT_ESTATE otherwise). */
NNT_API int32_t nnt_gpt2_block_adam(nnt_gpt2_block* blk, int32_t step, const nnt_adam_cfg* cfg);
/* SGD-with-momentum step on all 12 parameters; the velocities live in the slots
 * NNT_BLK_ADAM_M + parameter (the second-moment slots are not touched). */
NNT_API int32_t nnt_gpt2_block_sgd(nnt_gpt2_block* blk, const nnt_sgd_cfg* cfg);
/* bf16 blocks: (re)make the bf16 weight copies from the fp32 masters. */
NNT_API int32_t nnt_gpt2_block_sync_lowp(nnt_gpt2_block* blk);

/* acc[p] <- alpha * (gradient of parameter p) + acc[p] for the 12 parameters, as
 * 12 residual-add operations: gradient accumulation over micro-batches.  acc:
 * fp32 tensors shaped and tiled like the parameters (slot order). */
NNT_API int32_t nnt_gpt2_block_grads_axpy(nnt_gpt2_block* blk, float alpha, nnt_tensor* const* acc);

/* A chain of blocks as one flow of tasks (section 2: the whole training
 * iteration is submitted as one sequence of tasks and runs asynchronously):
 * acts[i] is the input of block i, acts[n_blocks] the output; dacts[i] is the
 * gradient with respect to acts[i] (dacts[n_blocks] is the input of backward).
 * All are [N_e, N_s, N_b] tensors of the blocks' dtype and tiling, owned by the
 * caller, as are the blocks.  Between nnt_capture_begin and nnt_capture_end the
 * three calls record the iteration of all blocks into one graph. */
typedef struct nnt_gpt2_stack nnt_gpt2_stack;
NNT_API int32_t nnt_gpt2_stack_create(nnt_ctx* ctx, int32_t n_blocks, nnt_gpt2_block* const* blocks,
                              nnt_tensor* const* acts, nnt_tensor* const* dacts, nnt_gpt2_stack** out);
NNT_API int32_t nnt_gpt2_stack_destroy(nnt_gpt2_stack* st);
NNT_API int32_t nnt_gpt2_stack_forward(nnt_gpt2_stack* st);
NNT_API int32_t nnt_gpt2_stack_backward(nnt_gpt2_stack* st);
NNT_API int32_t nnt_gpt2_stack_adam(nnt_gpt2_stack* st, int32_t step, const nnt_adam_cfg* cfg);

/* A GPT-2-shaped language model as one flow of tasks (section 3: embedding
 * layer, the blocks, layer normalization, linear head, Cross-Entropy loss,
 * optimizer): token and position embedding lookup and their sum, a chain of
 * blocks, the final layer norm, the head tied to the token embedding
 * (logits = W_te^T X_f), the loss summed over positions, the whole backward pass
 * and one Adam step on every parameter.  The caller creates the blocks and the
 * stack's activations as above, asks nnt_gpt2_model_slot for type, shape and
 * tiling of each of the model's own tensors, allocates them and hands them over;
 * the model keeps pointers, not ownership.
 *   parameters (fp32 masters): W_te [N_e, N_v] (one column per vocabulary item,
 *   tiled tile_e x tile_v), W_pe [N_e, N_s] (one column per position), gain and
 *   bias of the final layer norm [N_e]; + NNT_MDL_GRAD their gradients, +
 *   NNT_MDL_ADAM_M / _V their Adam moments; NNT_MDL_LOWP + {0, 1}: bf16 copies of
 *   W_te, W_pe (bf16 models only).
 *   activations: X_pos (position embeddings of the batch), X_f (final layer norm),
 *   dX_f, its statistics, the logits [N_v, N_s, N_b] (overwritten with their own
 *   gradient by the loss) and the loss's column statistics.
 * forward: tokens, positions, labels are device pointers to N_s * N_b int32
 * (position s + N_s * b of the batch); col_loss (N_s * N_b floats) and loss (1
 * float) are device buffers of the caller, valid after nnt_wait.  backward uses
 * the tokens / positions of the last forward call.  The gradient of W_te collects
 * the head's and the lookup's share; sums over positions that share a token use
 * hardware fp32 atomics (order not fixed). */
typedef struct nnt_gpt2_model nnt_gpt2_model;
enum {
    NNT_MDL_WTE = 0, NNT_MDL_WPE = 1, NNT_MDL_GAMMA_F = 2, NNT_MDL_BETA_F = 3,
    NNT_MDL_GRAD = 4, NNT_MDL_ADAM_M = 8, NNT_MDL_ADAM_V = 12, NNT_MDL_LOWP = 16,
    NNT_MDL_XPOS = 18, NNT_MDL_XF = 19, NNT_MDL_DXF = 20, NNT_MDL_STATS_F = 21, NNT_MDL_LOGITS = 22, NNT_MDL_LOSS_STATS = 23,
    NNT_MDL_NSLOTS = 24
};
NNT_API int32_t nnt_gpt2_model_slot(const nnt_gpt2_block_cfg* cfg, int64_t N_v, int64_t tile_v, int32_t slot, nnt_slot_info* out);
NNT_API int32_t nnt_gpt2_model_create(nnt_ctx* ctx, const nnt_gpt2_block_cfg* cfg, int64_t N_v, int64_t tile_v,
                              nnt_gpt2_stack* stack, nnt_tensor* const* slots, nnt_gpt2_model** out);
NNT_API int32_t nnt_gpt2_model_destroy(nnt_gpt2_model* m);
/* bf16 models: refreshes the bf16 copies of W_te, W_pe from the fp32 masters (after the caller wrote them) */
NNT_API int32_t nnt_gpt2_model_sync_lowp(nnt_gpt2_model* m);
NNT_API int32_t nnt_gpt2_model_forward(nnt_gpt2_model* m, const int32_t* tokens, const int32_t* positions,
                               const int32_t* labels, float* col_loss, float* loss);
NNT_API int32_t nnt_gpt2_model_backward(nnt_gpt2_model* m);
NNT_API int32_t nnt_gpt2_model_adam(nnt_gpt2_model* m, int32_t step, const nnt_adam_cfg* cfg);

NNT_API const char* nnt_version(void);

/* Measurement aid (no part of the method): launches `workgroups` workgroups of four
 * wavefronts that each issue `iters` x 8 matrix instructions back to back on operands held in
 * registers -- fp32 (32x32x2) or bf16 (32x32x16, fp32 accumulate) -- with no memory traffic.
 * random_operands != 0: operand registers hold pseudo-random values that differ from
 * instruction to instruction (as in a real product); 0: constants.  Timed by the caller (events
 * on `stream`), it gives the matrix-core rate that bounds the product kernels on the chip at
 * hand.  sink: device float the kernel practically never writes; flops_out (host, nullable):
 * flops issued by the launch. */
NNT_API int32_t nnt_probe_mfma_rate(void* stream, int32_t dtype, int32_t random_operands, int32_t iters,
                            int32_t workgroups, float* sink, double* flops_out);

#ifdef __cplusplus
}
#endif
#endif /* NNTILE_MI_H */
