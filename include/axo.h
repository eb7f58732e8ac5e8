/*
 * axo.h -- C ABI of the MI355X (gfx950) shard-GEMM library for 3D tensor-parallel
 * fully-connected layers.
 *
 * The operation (paper Section 3.2, "Three-dimensional Tensor Parallelism"; Figure 1;
 * Algorithm 1): an FC layer O = I x W with I in R^{m x k}, W in R^{k x n} is spread over a
 * virtual Gx x Gy x Gz grid of GPUs.  GPU g_{ix,iy,iz} holds one 2D block of I and one of W
 * and computes three local matrix products per layer:
 *
 *   forward  (Algorithm 1, forward function, local multiply)     Y_part  = X  . W
 *   dgrad    (Algorithm 1, backward function, first product)     dX_part = dY . W^T
 *   wgrad    (Algorithm 1, backward function, second product)    dW_part = X^T . dY
 *
 * The collectives that combine the partial results across GPUs are not part of this library;
 * it reproduces exactly one GPU's share of the work.
 *
 * Naming: T = m (tokens of one tensor-parallel group), K = k (in-features), N = n
 * (out-features), X = I, Y = O, dY = dL/dO, dX = dL/dI, dW = dL/dW.
 * Axis mapping: with transposed == 0 the reduction dimension K is split over Gx, N over Gy and
 * T over Gz; with transposed == 1 the roles of the X and Y axes are swapped (K over Gy, N over
 * Gx), which is the mapping of Algorithm 1 as printed and, per Section 3.2 ("Parallelizing an
 * entire network"), the one every second layer uses.  Local shard sizes are
 * M = T/Gz, Kl = K/G(k-axis), Nl = N/G(n-axis).
 *
 * Data: every matrix is row-major bf16 (bit patterns, 2 bytes per element) in DEVICE memory,
 * W stored [Kl x Nl] as the paper writes it.  Products accumulate in fp32 and are rounded once,
 * round-to-nearest-even, to bf16 at the store.  Leading dimensions are in elements and allow a
 * shard to be addressed in place inside a larger matrix.
 *
 * Ownership: the caller owns all buffers; the library allocates no device memory, keeps no pointer after
 * a call returns, and only enqueues work on the caller's HIP stream (no device synchronisation,
 * no host read-back).  Buffers must stay valid until the stream has executed the call.
 * The output of a product must not share a byte with an input of the same product (checked: AXO_ERR_BAD_ARG;
 * column blocks of one buffer that merely interleave are fine).  A matrix with no elements (a zero shard
 * dimension) is never dereferenced: its pointer may be NULL and its leading dimension is not checked.
 *
 * Errors: every function returns an int status, 0 on success, negative on error; nothing throws
 * or aborts.  All argument checks happen on the host before the first HIP call, so every status
 * except AXO_ERR_HIP can be produced without a GPU.  Host-side plan lists and per-shape plan caches
 * are the library's only allocations; when one fails the call returns AXO_ERR_NO_MEMORY and has
 * enqueued nothing or a prefix of its launches.
 */
#ifndef AXO_H
#define AXO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define AXO_VERSION 1

typedef enum axo_status {
    AXO_OK = 0,
    AXO_ERR_BAD_GRID = -1,     /* a grid dimension < 1                                           */
    AXO_ERR_BAD_COORD = -2,    /* coordinate outside the grid                                    */
    AXO_ERR_INDIVISIBLE = -3,  /* T, K or N not divisible by its grid dimension                  */
    AXO_ERR_NULL_PTR = -4,     /* a required pointer is NULL                                     */
    AXO_ERR_MISALIGNED = -5,   /* pointer not 16-byte aligned, or leading dimension not a        */
                               /* multiple of 8 elements                                         */
    AXO_ERR_BAD_LD = -6,       /* leading dimension smaller than the row length                  */
    AXO_ERR_WORKSPACE = -7,    /* workspace smaller than axo_workspace_bytes() asks for          */
    AXO_ERR_BAD_EPILOGUE = -8, /* unknown epilogue, or an epilogue with bias == NULL             */
    AXO_ERR_HIP = -9,          /* a HIP launch failed (the only status that needs a device)      */
    AXO_ERR_BAD_SIZE = -10,    /* T, K or N < 0, or a shard dimension beyond 2^31-1              */
    AXO_ERR_BAD_ARG = -11,     /* anything else malformed (unknown op, n_layers < 0, ...)        */
    AXO_ERR_NO_MEMORY = -12,   /* a host allocation of the library failed (plan lists, caches)   */
    AXO_ERR_TOO_LARGE = -13    /* more scratch needed than the allocation-free entry point holds */
} axo_status_t;

/* The problem statement of Section 3.2: grid, this GPU's coordinate, global sizes. */
typedef struct axo_problem {
    int32_t Gx, Gy, Gz; /* grid dimensions, each >= 1                                   */
    int32_t ix, iy, iz; /* this GPU is g_{ix,iy,iz}: 0 <= ix < Gx, and so on            */
    int64_t T, K, N;    /* GLOBAL tokens, in-features, out-features (each >= 0)         */
    int32_t transposed; /* 0: K over Gx, N over Gy.  1: K over Gy, N over Gx            */
    int32_t reserved;   /* must be 0                                                    */
} axo_problem_t;

/* Epilogue of the forward product.  Not part of the paper: the usual GPT MLP epilogue, fused
 * on the fp32 accumulator before the one rounding to bf16.
 * The bias vector is added only on shards whose coordinate along the axis that splits K is 0,
 * so that summing the partial products of that axis adds it exactly once.  The activation is
 * applied to this shard's (partial + bias); that equals the layer's activation only when the
 * K-splitting axis has size 1 (otherwise it is a kernel-shape measurement, since the true
 * activation must follow the all-reduce of Algorithm 1's forward function). */
typedef enum axo_epilogue {
    AXO_EPI_NONE = 0,
    AXO_EPI_BIAS = 1,           /* y + b                                                          */
    AXO_EPI_BIAS_GELU_TANH = 2, /* v = y + b;  0.5 v (1 + tanh( sqrt(2/pi) (v + 0.044715 v^3) ))  */
    AXO_EPI_BIAS_GELU_ERF = 3   /* v = y + b;  0.5 v (1 + erf( v / sqrt(2) ))                     */
} axo_epilogue_t;

typedef enum axo_op { AXO_OP_FWD = 0, AXO_OP_DGRAD = 1, AXO_OP_WGRAD = 2 } axo_op_t;

/* Library version (AXO_VERSION of the build). */
int axo_version(void);

/* Static, never NULL, human-readable text for a status code. */
const char *axo_status_string(int status);

/* Host only.  Validates the problem and derives this GPU's shard: local sizes M, Kl, Nl and the
 * offsets of its blocks in the global matrices (X block at [row0, k0], W block at [k0, n0],
 * Y / dY block at [row0, n0]).  Any output pointer may be NULL.
 * Errors: NULL_PTR (p), BAD_GRID, BAD_COORD, BAD_SIZE, INDIVISIBLE, BAD_ARG (reserved != 0 or
 * transposed not 0/1). */
int axo_shard_dims(const axo_problem_t *p, int64_t *M, int64_t *Kl, int64_t *Nl,
                   int64_t *row0, int64_t *k0, int64_t *n0);

/* Host only.  Bytes of device workspace the given op (axo_op_t) of this problem needs; 0 when
 * none.  The workspace holds fp32 partial sums when the reduction dimension is split inside one
 * GPU; it need not be initialised and may be reused by the next call on the same stream.
 * Returns 0 for an invalid problem (the op call itself reports the error). */
size_t axo_workspace_bytes(const axo_problem_t *p, int op);

/* Which kernels a product takes, as axo_fc_route reports it. */
typedef enum axo_route {
    AXO_ROUTE_NONE = 0,            /* an empty output: nothing is launched                                 */
    AXO_ROUTE_TILED = 1,           /* the tuned MFMA kernel, one launch                                    */
    AXO_ROUTE_COVERED = 2,         /* a ragged output covered with whole (overlapping) tuned tiles         */
    AXO_ROUTE_INTERIOR_STRIPS = 3, /* the interior on the tuned kernel, leftover strips on the general one */
    AXO_ROUTE_GENERAL = 4          /* the general (bounds-checked, untuned) kernel                         */
} axo_route_t;

/* Host only.  Reports in *route (axo_route_t) which kernels the product `op` (axo_op_t) of this
 * problem takes when its two inputs have leading dimensions ld_a, ld_b (in the argument order of the
 * product's entry point: X, W for forward; dY, W for dgrad; X, dY for wgrad) and its output ld_out.
 * The choice depends on the shard shape and on the leading dimensions only (the tuned kernel forms
 * 32-bit byte offsets inside an operand tile), never on data.  For capacity planning and tests.
 * Errors: those of the product's argument checks; NULL_PTR (route); BAD_ARG (unknown op). */
int axo_fc_route(const axo_problem_t *p, int op, int64_t ld_a, int64_t ld_b, int64_t ld_out, int *route);

/* Forward local product  Y[M x Nl] = epilogue( X[M x Kl] . W[Kl x Nl] ).
 * X, W, Y: device pointers, bf16, row-major, 16-byte aligned; ldx >= Kl, ldw >= Nl, ldy >= Nl,
 * each a multiple of 8.  bias: device pointer to Nl bf16 values (16-byte aligned) or NULL when
 * epilogue == AXO_EPI_NONE.  ws / ws_bytes: device workspace of at least
 * axo_workspace_bytes(p, AXO_OP_FWD) bytes (may be NULL when that is 0).  hip_stream: a
 * hipStream_t (NULL = the default stream).  A shard with M, Kl or Nl == 0 is valid: with
 * Kl == 0 the output is epilogue(0); with M or Nl == 0 nothing is written.
 * Errors: those of axo_shard_dims; BAD_EPILOGUE (unknown epilogue, or one with bias == NULL);
 * NULL_PTR, BAD_LD, MISALIGNED for X, W, Y, bias; BAD_ARG (Y shares bytes with X, W or bias); WORKSPACE;
 * HIP; NO_MEMORY.
 * Speed: the tuned kernel takes shards whose reduction length (Kl here, Nl for dgrad) is a multiple of 8 and
 * whose output has at least 256 rows and 128 columns, the column count a multiple of 8; leading dimensions
 * that are multiples of 64 elements keep every 128-byte row segment inside one cache line (worth 10-20 %).
 * Everything else is computed by a general kernel that is several times slower; axo_fc_route tells which. */
int axo_fc_fwd(const axo_problem_t *p, const void *X, int64_t ldx, const void *W, int64_t ldw,
               const void *bias, int epilogue, void *Y, int64_t ldy,
               void *ws, size_t ws_bytes, void *hip_stream);

/* Backward data gradient  dX[M x Kl] = dY[M x Nl] . W[Kl x Nl]^T.
 * lddy >= Nl, ldw >= Nl, lddx >= Kl; same alignment rules; workspace per AXO_OP_DGRAD.
 * Errors: as axo_fc_fwd, without BAD_EPILOGUE. */
int axo_fc_dgrad(const axo_problem_t *p, const void *dY, int64_t lddy, const void *W, int64_t ldw,
                 void *dX, int64_t lddx, void *ws, size_t ws_bytes, void *hip_stream);

/* Backward weight gradient  dW[Kl x Nl] = X[M x Kl]^T . dY[M x Nl].
 * ldx >= Kl, lddy >= Nl, lddw >= Nl; same alignment rules; workspace per AXO_OP_WGRAD.
 * Errors: as axo_fc_fwd, without BAD_EPILOGUE. */
int axo_fc_wgrad(const axo_problem_t *p, const void *X, int64_t ldx, const void *dY, int64_t lddy,
                 void *dW, int64_t lddw, void *ws, size_t ws_bytes, void *hip_stream);

/* ---- The steps either side of the three products in a layer's backward pass ------------------
 * They are not part of the paper's Algorithm 1 (which stops at the products) but every layer of
 * the networks it trains has them; mixed precision as in Section 6.1 (bf16 data, fp32 master
 * gradients).  Like the forward epilogue they are applied to THIS GPU's partial result, which is
 * the layer's true value only when the group that the product is reduced over has size 1. */

/* Data gradient taken through the activation of the layer below:
 *   dX[M x Kl] = (dY[M x Nl] . W[Kl x Nl]^T) * act'(pre[M x Kl]),
 * pre = that layer's bf16 pre-activation (bias included), act = AXO_EPI_BIAS_GELU_TANH or
 * AXO_EPI_BIAS_GELU_ERF (selects which GELU's derivative; no bias is involved).  The multiply
 * happens on the fp32 accumulator, before the one rounding to bf16.  ldpre >= Kl; otherwise the
 * rules of axo_fc_dgrad.  Errors: those of axo_fc_dgrad, BAD_EPILOGUE for any other act. */
int axo_fc_dgrad_act(const axo_problem_t *p, const void *dY, int64_t lddy, const void *W, int64_t ldw,
                     const void *pre, int64_t ldpre, int act, void *dX, int64_t lddx,
                     void *ws, size_t ws_bytes, void *hip_stream);

/* Weight gradient accumulated in fp32:  dW[Kl x Nl] += X[M x Kl]^T . dY[M x Nl], dW a device
 * matrix of fp32 (the master gradient), lddw in fp32 elements, >= Nl and a multiple of 4, dW
 * 16-byte aligned.  The product is added unrounded; each element is updated by exactly one
 * workgroup, so the result does not depend on scheduling.  Otherwise the rules of axo_fc_wgrad. */
int axo_fc_wgrad_acc(const axo_problem_t *p, const void *X, int64_t ldx, const void *dY, int64_t lddy,
                     float *dW, int64_t lddw, void *ws, size_t ws_bytes, void *hip_stream);

/* Bias gradient: db[n] = sum over the M local rows of dY[t, n] (accumulate == 0) or db[n] += that
 * sum (accumulate == 1); db: Nl fp32 values in device memory, 4-byte aligned.  fp32 sums in a
 * fixed order (no atomics).  Errors: problem errors, NULL_PTR, BAD_LD, MISALIGNED, BAD_ARG
 * (accumulate not 0/1), HIP. */
int axo_bias_grad(const axo_problem_t *p, const void *dY, int64_t lddy, float *db, int accumulate,
                  void *hip_stream);

/* Host only.  Bytes of device workspace axo_bias_grad_ws needs for this problem (0 for shards so
 * small that it does not split their rows, and for an invalid problem). */
size_t axo_bias_grad_workspace_bytes(const axo_problem_t *p);

/* The bias gradient of axo_bias_grad, with the rows of dY split over several workgroups per
 * 64-column strip: a 6144-column shard gives axo_bias_grad 96 workgroups for 256 compute units, which
 * leaves it bound by memory latency; this form keeps about four workgroups per unit in flight.  Every
 * workgroup writes the fp32 sums of its row slice to the workspace, and the one that finishes last
 * adds the slices of its strip in ascending order: no floating-point atomics, so the result is a fixed
 * function of the input (equal from run to run; it differs from axo_bias_grad's in the last bits,
 * the rows being summed in another order).
 * ws: device memory, 16-byte aligned, at least axo_bias_grad_workspace_bytes(p) bytes (may be NULL
 * when that is 0).  It begins with one arrival counter per strip, which must be ZERO when the call
 * starts executing and is zero again when it has finished: zero-fill the workspace once after
 * allocating it and leave it to calls of this function.  Calls that share a workspace must not overlap
 * in time (same stream, or ordered by events).
 * Errors: those of axo_bias_grad; WORKSPACE (ws NULL or too small); MISALIGNED (ws). */
int axo_bias_grad_ws(const axo_problem_t *p, const void *dY, int64_t lddy, float *db, int accumulate,
                     void *ws, size_t ws_bytes, void *hip_stream);

/* axo_bias_grad_ws for callers that cannot allocate device memory or pass a workspace along: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernel, same
 * slicing, same bits as axo_bias_grad_ws; the slice sums and arrival counters live in a fixed array
 * of axo_bias_grad_static_limit() bytes (256 KiB) inside the library's device image instead of a
 * workspace.  Each GPU the library runs on holds its own copy of that array from the first use to
 * the end of the process.  The call allocates nothing (no hipMalloc, no hipFree, no host
 * containers); on its first use on a device it asks the runtime once for the array's address there.
 * The array is shared by all calls on a GPU and keeps their contents: the counters are zero when
 * the library is loaded and every call returns them to zero, the slice sums need no clearing.  Two
 * calls that overlap in time on one GPU (different streams without an ordering) race on it.  The address
 * lookup is not a stream operation; make the first call on a device outside any stream capture.
 * Errors: those of axo_bias_grad; TOO_LARGE when axo_bias_grad_workspace_bytes(p) exceeds the limit
 * (with today's slicing no shape needs more than 132 KiB, so none is refused); HIP. */
int axo_bias_grad_static(const axo_problem_t *p, const void *dY, int64_t lddy, float *db, int accumulate,
                         void *hip_stream);

/* Host only.  Size in bytes of the fixed scratch array of axo_bias_grad_static. */
size_t axo_bias_grad_static_limit(void);

/* One FC layer of a chain: its problem, epilogue, and the caller's buffers with their leading
 * dimensions.  X and W are kept by the caller between forward and backward (the cache of
 * Algorithm 1's forward function).  dY is the gradient with respect to the layer's output
 * before the activation. */
typedef struct axo_layer {
    axo_problem_t p;
    int32_t epilogue; /* axo_epilogue_t */
    int32_t reserved; /* must be 0      */
    const void *X;    int64_t ldx;
    const void *W;    int64_t ldw;
    const void *bias;           /* NULL unless epilogue != AXO_EPI_NONE */
    void *Y;          int64_t ldy;
    const void *dY;   int64_t lddy;
    void *dX;         int64_t lddx;
    void *dW;         int64_t lddw;
} axo_layer_t;

/* Host only.  Largest workspace any single product of the chain needs. */
size_t axo_layer_step_workspace_bytes(const axo_layer_t *layers, int n_layers);

/* The 3 * n_layers local products of Algorithm 1 for a chain of layers, with the results of this
 * program order: forward of layers 0..n-1, then for layers n-1..0 dgrad followed by wgrad (Section
 * 4.1 issues the dgrad all-reduce before computing wgrad, which fixes that order), all enqueued on
 * one stream without host synchronisation.
 *
 * The library does not simply launch them one after the other.  It compares the byte ranges the
 * products read and write (first to last element of every matrix; pointers are compared, never
 * dereferenced), gives every product a dependence level (0: conflicts with no earlier product;
 * otherwise one more than the highest level among the earlier products whose output it reads or
 * overwrites, or whose input it overwrites), and enqueues level by level.  The products of one
 * level are independent, and those the tiled kernel takes share grouped launches: the output
 * tiles of up to 12 products in one grid, most expensive tiles first, so that products too small
 * to fill the GPU on their own (a 1536 x 1536 shard is 36 tiles for 256 compute units) run side by
 * side and the level pays one ramp-up and one tail instead of one per product.  A chain whose
 * layers have buffers of their own is a single level; a layer whose X is the previous layer's Y,
 * or whose dX is the previous layer's dY, lands on the next level; dgrad and wgrad of a layer
 * always share a level.  Results are the same, bit for bit, whatever the grouping (every output
 * element is accumulated in the same order in every tile shape).  Two column blocks interleaved
 * in one buffer count as overlapping, which only costs concurrency.  Chains of more than 256
 * layers are not analysed and keep the program order, one product per launch.
 * All layers are validated before the first launch; on a validation error nothing is enqueued. */
int axo_layer_step(const axo_layer_t *layers, int n_layers, void *ws, size_t ws_bytes,
                   void *hip_stream);

/* The same products in the same program order, one launch per product and nothing else: the plain
 * reading of the order above, kept for comparison (results are bit-identical to axo_layer_step's)
 * and for timing what the dependence analysis and the grouped launches gain. */
int axo_layer_step_ordered(const axo_layer_t *layers, int n_layers, void *ws, size_t ws_bytes,
                           void *hip_stream);

/* Host only.  The dependence levels axo_layer_step would use: *n_levels receives their number
 * (0 for an empty chain) and, when levels is not NULL, levels[0 .. 3 * n_layers) the level of
 * every product in program order (forward of layers 0..n-1, then dgrad, wgrad of layers n-1..0).
 * Errors: those of axo_layer_step's validation (with ws = NULL, ws_bytes = 0), NULL_PTR (n_levels). */
int axo_layer_step_levels(const axo_layer_t *layers, int n_layers, int *n_levels, int *levels);

/* ---- A layer's whole local step, backward-side extras included ----------------------------
 * One FC layer as axo_layer_t describes it, plus what its backward pass does besides the two
 * products (see axo_fc_dgrad_act, axo_fc_wgrad_acc, axo_bias_grad for the operations and their
 * argument rules).  Every extra is optional and switched on by a non-NULL pointer:
 *   pre   != NULL: dX = (dY . W^T) * act'(pre), act = act_below (AXO_EPI_BIAS_GELU_TANH or _ERF);
 *                  with pre == NULL act_below must be 0 and dgrad is the plain product;
 *   dW32  != NULL: the weight gradient is accumulated, unrounded, into this fp32 matrix
 *                  (dW32 += X^T . dY, lddw32 in fp32 elements) and layer.dW is not written
 *                  (it may be NULL);
 *   db    != NULL: db[Nl] = column sums of dY in fp32 (db += ... when accumulate_db == 1). */
typedef struct axo_layer_ext {
    axo_layer_t layer;
    const void *pre;  int64_t ldpre;   /* [M x Kl] bf16 pre-activation of the layer below, or NULL */
    float *dW32;      int64_t lddw32;  /* [Kl x Nl] fp32 master gradient, or NULL                  */
    float *db;                         /* [Nl] fp32 bias gradient, or NULL                         */
    int32_t act_below;                 /* axo_epilogue_t, see above                                */
    int32_t accumulate_db;             /* 0 or 1                                                   */
} axo_layer_ext_t;

/* axo_layer_step for layers with extras.  Program order: forward of layers 0..n-1, then for
 * layers n-1..0 dgrad, wgrad, bias gradient.  Scheduling is that of axo_layer_step: dependence
 * levels from the byte ranges read and written (an accumulating call reads what it writes),
 * independent products of a level in grouped launches (the fused variants take part in them: they
 * differ from the plain products only in their epilogue).  A bias gradient of at least 4033
 * columns (the width from which the stand-alone call uses 64-column strips) rides along in its
 * level's last grouped launch as a segment of memory-bound workgroups; narrower ones are launches
 * of their own within their level.  Results are bit-identical to the single calls in program order.
 * Errors: those of the single calls; BAD_EPILOGUE (act_below not a GELU kind with pre != NULL, or
 * not 0 with pre == NULL); BAD_ARG (accumulate_db not 0/1, a reserved field not 0, n_layers < 0 or
 * > 4096).  On a validation error nothing is enqueued. */
int axo_layer_step_ext(const axo_layer_ext_t *layers, int n_layers, void *ws, size_t ws_bytes,
                       void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* AXO_H */
