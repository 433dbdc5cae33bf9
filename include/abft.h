/*
 * abft.h -- C ABI of the ABFT-protected matrix-multiplication library for MI355X (gfx950).
 *
 * The library computes C = A.B for the linear layers of neural-network inference
 * (fully-connected layers and convolutions lowered to a matrix product) and checks
 * the result with algorithm-based fault tolerance, following Kosaian & Rashmi,
 * "Arithmetic-Intensity-Guided Fault Tolerance for Neural Network Inference on
 * GPUs" (SC '21).  Notation is the paper's (Sec. 2.1): A is M x K (activations),
 * B is K x N (weights, known before inference), C is M x N.
 *
 * General conventions
 *  - Every matrix / vector pointer is a DEVICE pointer owned by the caller unless
 *    the parameter says "host".  The library allocates device memory only inside a
 *    plan (abft_plan_create), released by abft_plan_destroy.
 *  - All work is enqueued asynchronously on the HIP stream passed as `stream`
 *    (a hipStream_t cast to void*, NULL = the default stream).  Results, the fault
 *    flag and the report are valid once that stream has been synchronised.
 *  - Functions returning int return ABFT_OK (0) or a negative ABFT_E_* code.  They
 *    never abort and never throw.  A detected fault is NOT an error return: C is
 *    always written (the method detects, it does not correct; Sec. 2.3) and the
 *    fault flag is raised.
 *  - Leading dimensions are in elements.  Operands may have any alignment and any
 *    leading dimension; 16-byte aligned pointers with K and the leading dimensions
 *    multiples of 16 bytes take the fast vectorised path.
 *  - Thread safety: calls on different streams with different workspaces, flags and
 *    reports do not interfere.
 */
#ifndef ABFT_H
#define ABFT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- error codes -------------------------------------------------------- */
#define ABFT_OK 0
#define ABFT_E_NULL (-1)       /* a required pointer is NULL */
#define ABFT_E_SHAPE (-2)      /* M, N or K <= 0, or a convolution geometry with no output */
#define ABFT_E_LD (-3)         /* a leading dimension is smaller than the row length */
#define ABFT_E_ENUM (-4)       /* unknown dtype / mode / layout value */
#define ABFT_E_WORKSPACE (-5)  /* workspace missing, misaligned (256 B) or too small */
#define ABFT_E_INJECT (-6)     /* fault descriptor out of range */
#define ABFT_E_HIP (-7)        /* a HIP runtime call failed (launch, allocation) */
#define ABFT_E_PLAN (-8)       /* bad plan handle or layer index */
#define ABFT_E_UNSUPPORTED (-9) /* the scheme is not available for this product (see ABFT_GLOBAL_WEIGHTED) */

/* ---- enums --------------------------------------------------------------- */
/* Protection scheme.  GLOBAL: kernel-level ABFT (Sec. 2.4-2.5): the weight checksums are
 * formed offline, the output summation is fused into the product kernel's epilogue and
 * compared there with the dot product of activation and weight checksums -- per workgroup
 * tile of C, so for a product that fits one tile this is the single whole-matrix
 * comparison.  For 16-byte aligned operands the product kernel forms that dot product
 * itself from the A tiles it loads (one kernel in all); otherwise, and for very large
 * products, an activation-checksum kernel runs first.  THREAD: the paper's one-sided
 * thread-level scheme (Sec. 5.2.2), carried out per wavefront register tile.  AUTO:
 * whatever abft_select returns (intensity-guided ABFT, Sec. 5.3). */
typedef enum {
    ABFT_NONE = 0,
    ABFT_GLOBAL = 1,   /* global ABFT, one comparison per workgroup tile (Sec. 2.4, 2.5) */
    ABFT_THREAD = 2,   /* one-sided thread-level ABFT, one comparison per wavefront tile (Sec. 5.2) */
    ABFT_AUTO = 3,     /* abft_select decides between GLOBAL and THREAD (Sec. 5.3) */
    /* Thread-level replication with single accumulation (Sec. 5.1), the baseline the paper weighs
     * one-sided ABFT against: every MFMA of the product is issued a second time, all those of one A
     * fragment into one accumulator block, whose sum must equal the sum of the wavefront tile.
     * Same tiles, comparisons, tolerance, report and k partition as ABFT_THREAD; never chosen by
     * ABFT_AUTO or by a plan's profile. */
    ABFT_REPLICA = 4,
    /* One-sided thread-level ABFT with the tile checksum of B_t added up in the operand type, as the
     * paper does it (Sec. 5.2.2: packed half-precision adds): one extra MFMA per A fragment and k
     * step (Table 1's M_t / 2) and one packed add per further B fragment.  The roundings of those
     * adds (2^-11 per add in F16, 2^-8 in BF16) widen the tolerance (abft_tolerance_half_coeff):
     * faults smaller than about an rms of C in one element go unseen.  ABFT_THREAD keeps the
     * checksum exact instead, at twice (BF16: three times) the extra MFMAs. */
    ABFT_THREAD_HALF = 5,
    /* Two-sided thread-level ABFT (Sec. 5.2.1, Table 1 middle column): checksums of both the A
     * fragments and the B fragments of the wavefront tile, added up in the operand type, one extra
     * MFMA per k step.  Same tolerance rule as ABFT_THREAD_HALF with both sides' adds. */
    ABFT_TWOSIDED = 6,
    /* (I8 has no sums in the operand type: ABFT_THREAD_HALF and ABFT_TWOSIDED run as ABFT_THREAD.
     * Neither is chosen by ABFT_AUTO or by a plan's profile.) */
    /* Global ABFT with several independent checksums (Sec. 2.4, last paragraph): per workgroup tile
     * three comparisons -- the plain one, one with the tile's rows weighted, one with its columns
     * weighted (I8: weights i + 1, j + 1; F16: (i + 1) / region_m, (j + 1) / region_n) -- each with
     * the global scheme's tolerance on the weighted tile.  Two wrong elements whose errors cancel in
     * the plain sum are still seen unless they share a row and a column; a single wrong element is
     * located (abft_report_t.fault_row / fault_col / fault_delta).  The extra checksums ride in spare
     * columns of an extra matrix operand, so the scheme exists where that operand does: products
     * that run on the latency-bound tiling (up to a few hundred output tiles of at most 64 x 64;
     * abft_region_shape tells) with F16 or I8 operands; elsewhere the call returns
     * ABFT_E_UNSUPPORTED.  Workspace, beta and report as for ABFT_GLOBAL. */
    ABFT_GLOBAL_WEIGHTED = 7
} abft_mode_t;
/* Activation function a layer applies to its output as it is stored (Sec. 2.4 step 4). */
typedef enum { ABFT_ACT_NONE = 0, ABFT_ACT_RELU = 1 } abft_act_t;

/* Operand type.  F16 / BF16: A, B and C are fp16 / bf16, accumulation in fp32.
 * I8: A and B are int8, C is int32, accumulation in int32 (exact). */
typedef enum { ABFT_F16 = 0, ABFT_BF16 = 1, ABFT_I8 = 2 } abft_dtype_t;

/* Storage order of the weight matrix B.
 *  ABFT_B_NK: element B[k][n] is at B[n*ldb + k]  (each output channel's K weights
 *             contiguous -- the order inference frameworks keep linear / NHWC conv
 *             weights in; the fast path).
 *  ABFT_B_KN: element B[k][n] is at B[k*ldb + n]  (row-major K x N). */
typedef enum { ABFT_B_NK = 0, ABFT_B_KN = 1 } abft_blayout_t;

/* ---- small structs -------------------------------------------------------- */
/* Test hook for the fault model of Sec. 2.3 (one wrong value in C caused by
 * processing logic): flip bit `bit` (0..31) of the fp32 / int32 accumulator of
 * element (row, col).
 *   k_after = -1: the finished accumulator is flipped just before the checksum epilogue.
 *   k_after >= 0: the running accumulator is flipped once the products with k < k_after have
 *     been added (must be a positive multiple of the k_step reported by abft_tile_shape and
 *     < K); the corruption then stays until the end of the loop.
 *   k_after = -2: the finished value is flipped after the partial sums of the wavefronts that
 *     share a register tile (abft_k_ways) have been added, just before the checks and the store
 *     read it; the same as -1 where one wavefront forms the whole sum.
 * When several wavefronts share a register tile along k (abft_k_ways), the running accumulator
 * is that of the wavefront holding k_after - 1, and k_after = -1 flips the finished partial
 * accumulator of the wavefront holding K - 1.
 * Convolutions: row = output pixel, col = output channel; k counts in the order of abft_conv_t
 * (a call with k_after >= 0 runs without the lowering to row segments). */
typedef struct {
    int64_t row, col;
    int32_t bit;
    int32_t k_after;
} abft_fault_t;

/* Convolution geometry for the implicit-GEMM path.  Activations are NHWC
 * (batch, H, W, Cin) dense; the lowered problem has M = batch*OH*OW,
 * K = KH*KW*Cin with k = (kh*KW + kw)*Cin + c, and N = output channels. */
typedef struct {
    int32_t batch, H, W, Cin;
    int32_t KH, KW, stride, pad;
} abft_conv_t;

/* What the checksum comparisons saw; optional diagnostics written by the device.
 * Both schemes make one comparison per region of C: GLOBAL per workgroup tile
 * (abft_region_shape), THREAD per wavefront register tile (abft_tile_shape).
 * lhs = output summation of the region with the largest |lhs - rhs| / tau seen,
 * rhs = its checksum product, tau = its tolerance, worst_ratio = that ratio (0 when
 * tau = 0 and both sides are equal, +inf when they differ or are not finite); ties go to
 * the region with the lowest index.  tiles = number of comparisons made.  Must be zero-filled by the caller before the call. */
typedef struct {
    double lhs, rhs, tau, worst_ratio;
    uint64_t tiles;
    double frob, l1;   /* ||C_S||_F and sum |C_ij| of the region lhs/rhs/tau belong to (l1: GLOBAL only) */
    uint32_t lock;     /* used by the device while it updates the block */
    uint32_t region;   /* 1 + row-major index of that region in the partition of C into regions (edge regions clipped) */
    /* ABFT_GLOBAL_WEIGHTED only (else left as the caller set them): where a single wrong element of
     * the reported region would sit, from the ratios of the weighted residuals to the plain one
     * (-1, -1 when the plain comparison held or the ratios point outside the region), by how much
     * the region's sum is off, and residual / tolerance of the two weighted comparisons
     * (worst_ratio is then the largest of the three). */
    int32_t fault_row, fault_col;
    double fault_delta, ratio_rows, ratio_cols;
} abft_report_t;

/* ---- the protected product ------------------------------------------------ */
/*
 * C = A.B with the checks of `mode` (Sec. 2.4 / 5.2.2 / 5.3).
 *   A   : M x K row-major, lda >= K.
 *   B   : K x N in the order `b_layout` says, ldb >= K (NK) or >= N (KN).
 *   C   : M x N row-major, ldc >= N; fp16 / bf16 (rounded to nearest even from the
 *         fp32 accumulators) or int32.
 *   beta: optional weight checksums made earlier by abft_weight_checksum with block_n =
 *         the region_n of abft_region_shape for this problem (a buffer of abft_beta_bytes).
 *         Used by GLOBAL only; NULL makes the call compute them into the
 *         workspace first.  THREAD never
 *         reads it: it recomputes tile-local weight checksums in registers (Sec. 5.2.1).
 *   workspace / workspace_bytes: scratch of at least abft_workspace_bytes(...) bytes,
 *         256-byte aligned; may be NULL when that size is 0.  Only GLOBAL uses one (partial
 *         checksum dot products; the weight checksums when `beta` is NULL).  Its contents
 *         need no initialisation and mean nothing after the call; calls that share a
 *         workspace must be ordered on one stream.
 *   fault_flag: device uint32, OR-ed with 1 when a comparison fails.  The caller
 *         zeroes it.  May be NULL only for ABFT_NONE.
 *   report: optional device abft_report_t (zero-filled by the caller), else NULL.
 *   inject: optional HOST pointer to a fault to plant (testing), else NULL.
 */
int abft_gemm(int M, int N, int K, const void *A, int64_t lda, const void *B, int64_t ldb,
              int b_layout, void *C, int64_t ldc, int dtype, int mode, const void *beta,
              void *workspace, size_t workspace_bytes, uint32_t *fault_flag, abft_report_t *report,
              const abft_fault_t *inject, void *stream);

/* abft_gemm for callers that cannot allocate device memory or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and
 * results as abft_gemm without `workspace`: the global scheme's scratch (partial checksum dot
 * products; the weight checksums when `beta` is NULL) lives in an array of
 * abft_static_scratch_bytes() bytes (8 MiB) inside the library, one copy per GPU the library
 * runs on, held until the process ends.  The call allocates nothing.  A product that needs more
 * scratch than that (beyond about 8192^3 with `beta` given) returns ABFT_E_WORKSPACE and
 * launches nothing.  Nothing in the array needs to be zero: every byte a call reads was written
 * earlier in the same call.  All calls on one GPU share its array, so calls that may overlap
 * there (different streams, different host threads) race: order them on one stream.  The first
 * call on a device looks the array's address up (not a stream operation: make that call outside
 * graph capture). */
int abft_gemm_static(int M, int N, int K, const void *A, int64_t lda, const void *B, int64_t ldb,
                     int b_layout, void *C, int64_t ldc, int dtype, int mode, const void *beta,
                     uint32_t *fault_flag, abft_report_t *report, const abft_fault_t *inject,
                     void *stream);
/* Size of that array in bytes. */
size_t abft_static_scratch_bytes(void);

/* Same for a convolution executed as an implicit matrix product (Sec. 2.1): x is
 * the NHWC activation tensor; B holds the filters as the K x N matrix described at
 * abft_conv_t; C is (batch*OH*OW) x N row-major, i.e. the NHWC output. */
int abft_conv(const abft_conv_t *conv /* host */, int N, const void *x, const void *B, int64_t ldb,
              int b_layout, void *C, int64_t ldc, int dtype, int mode, const void *beta,
              void *workspace, size_t workspace_bytes, uint32_t *fault_flag, abft_report_t *report,
              const abft_fault_t *inject, void *stream);

/* Bytes of workspace abft_gemm / abft_conv want for this problem (0 when none is used). */
size_t abft_workspace_bytes(int M, int N, int K, int dtype, int mode);

/* The same for a convolution, given its geometry (conv: host).  A convolution whose channel
 * count does not fill 16-byte chunks (an RGB first layer) runs several times faster when the
 * workspace has this size: the call then copies the input once with its zero border and
 * re-orders the weights (both into the workspace) so that the product can read whole chunks.
 * With a workspace of only abft_workspace_bytes the same call gathers element by element.
 * The lowered product multiplies the few input values that follow each window's run in its
 * input row (and, in the last k tile, rows below the window) by zero weights: it assumes finite
 * activations.  A non-finite activation then also turns outputs of neighbouring windows into
 * NaN; a protected scheme raises the flag in either form (a non-finite sum fails). */
size_t abft_conv_workspace_bytes(const abft_conv_t *conv /* host */, int N, int dtype, int mode);

/* Offline weight checksums (Sec. 2.5), one per block of block_n consecutive columns: with
 * nb = ceil(N / block_n), beta_b[k] = sum over n in [b*block_n, min(N, (b+1)*block_n)) of B[k][n].
 * The buffer `beta` (device, abft_beta_bytes(K, N, block_n) bytes, 256-byte aligned) receives four
 * copies: first K x nb values k-major, beta[k*nb + b], as doubles (F16 / BF16) or int64 (I8);
 * then, at the next multiple of 256 bytes, the copy the product kernels read inside their loops
 * (4 bytes per k and block): per block b, K floats (F16 / BF16), or K low digits followed by K
 * high digits, one signed byte each, beta_b[k] = lo + 256 hi (I8; exact for block_n <= 256);
 * then, again at the next multiple of 256 bytes, 8 bytes per k and block for the matrix-unit form
 * of the latency-bound tiling: F16: per block four planes of K halves, fl16(beta),
 * fl16((beta - fl16(beta)) 2^11) and the same two pieces of the column-weighted checksum
 * sum_j (j + 1) / block_n * B[k][b*block_n + j] (block_n as passed, also where N is smaller); I8: per block four planes of K signed bytes, the
 * digits (base 256, balanced, least significant first) of sum_j (j + 1) * B[k][b*block_n + j];
 * last, again at a multiple of 256 bytes, per block and per k tile of the large-tile kernel (64
 * values of k; I8: 128) one record of 1 KB that the kernel copies in with its operand tiles: F16:
 * 64 halves fl16(beta), 64 halves fl16((beta - fl16(beta)) 2^11), then from byte 256 the 64 floats;
 * BF16: the 64 floats at byte 256; I8: 128 low digits, 128 high digits.
 * block_n <= 0 or >= N gives the plain K-vector B.1 . */
int abft_weight_checksum(int K, int N, const void *B, int64_t ldb, int b_layout, int dtype, int block_n,
                         void *beta, void *stream);

/* Size in bytes of the buffer abft_weight_checksum fills (0 for invalid arguments). */
size_t abft_beta_bytes(int K, int N, int block_n);

/* Activation checksum (Sec. 2.4 step 1): alpha[k] = sum_m A[m][k] as K doubles / int64.
 * `conv` (host, may be NULL) makes A the lowered matrix of the NHWC tensor passed as A. */
int abft_activation_checksum(int M, int K, const void *A, int64_t lda, const abft_conv_t *conv, int dtype,
                             void *alpha, void *stream);

/* ---- selector (Sec. 3.1 Eq. 1, Sec. 5.3) ---------------------------------- */
/* FLOPs / bytes with FLOPs = 2MNK and bytes = sA*M*K + sB*K*N + sC*M*N for the
 * storage sizes of `dtype` (2,2,2 for F16/BF16; 1,1,4 for I8); unpadded dimensions. */
double abft_arithmetic_intensity(int M, int N, int K, int dtype);
/* Compute-to-memory-bandwidth ratio used for `dtype`: dense MFMA peak over HBM
 * bandwidth of MI355X (2516.6 TFLOP/s resp. 5033.2 TOP/s over 8 TB/s) unless
 * overridden by abft_set_cmr. */
double abft_cmr(int dtype);
/* Override the ratio (e.g. with a measured one); value <= 0 restores the default. */
void abft_set_cmr(int dtype, double value);
/* ABFT_GLOBAL if the layer is compute bound by Eq. 1 (intensity > CMR, strictly),
 * else ABFT_THREAD.  Negative error code on bad arguments. */
int abft_select(int M, int N, int K, int dtype);

/* Register-tile partition the THREAD scheme uses for this problem: C is cut into
 * tile_m x tile_n tiles starting at (0,0) (edge tiles clipped), one comparison each.
 * `aligned` is non-zero when every operand pointer and leading dimension (and K, or
 * Cin for a convolution) is a multiple of 16 bytes, which makes the largest tile
 * eligible.  k_step is the granularity of abft_fault_t.k_after.  Any of the outputs
 * may be NULL. */
int abft_tile_shape(int M, int N, int K, int dtype, int aligned, int *tile_m, int *tile_n, int *k_step);

/* Workgroup tiling of C: the GLOBAL scheme makes one comparison per region_m x region_n
 * block of C (edge blocks clipped) and wants its weight checksums per block of region_n
 * columns.  `aligned` as for abft_tile_shape. */
int abft_region_shape(int M, int N, int K, int dtype, int aligned, int *region_m, int *region_n);

/* Split along k inside a workgroup (latency-bound products): `ways` wavefronts share each
 * register tile, wavefront w multiplying the k with (k / step) % ways == w; their partial
 * tiles are added in wavefront order at the end (bit-reproducible) and every scheme makes its
 * comparison on the added-up tile, so the split only matters for where an injected fault
 * lands (abft_fault_t).  ways = 1: not split. */
int abft_k_ways(int M, int N, int K, int dtype, int aligned, int mode, int *ways, int *step);

/* Comparison tolerance (the paper states none; Sec. 2.4 step 4 says "compare").  A comparison
 * covers a region C_S of C -- one workgroup tile (abft_region_shape) for GLOBAL, one wavefront
 * register tile (abft_tile_shape) for THREAD / REPLICA -- and passes when
 *     |lhs - rhs| <= tau = coeff * ||C_S||_F + bias_coeff * sum_{S} |C_ij|
 * with both norms taken from the fp32 accumulators.
 *   coeff      = 8 * (2^-24 * sqrt(K) + u): random-walk rounding of K fp32 accumulations per
 *                entry, added in quadrature over the region, times a safety factor of 8;
 *                u = 0 for GLOBAL, 2^-22 (F16) / 2^-23 (BF16) for THREAD and REPLICA
 *                (precision of the in-register tile checksum).
 *   bias_coeff = 1e-3 * 2^-24 * K for GLOBAL (a same-sign drift of the accumulation that adds
 *                linearly over a region of same-sign entries), 0 otherwise.
 * ABFT_THREAD_HALF / ABFT_TWOSIDED add abft_tolerance_half_coeff(...) to coeff.
 * I8 compares exactly: both are 0.  A non-finite side always fails.
 * abft_tolerance_coeff returns coeff, abft_tolerance_bias_coeff returns bias_coeff. */
double abft_tolerance_coeff(int K, int dtype, int mode);
double abft_tolerance_bias_coeff(int K, int dtype, int mode);
/* Further coefficient of ||C_S||_F for ABFT_THREAD_HALF and ABFT_TWOSIDED on wavefront tiles of
 * tile_m x tile_n (abft_tile_shape): 4 * u_half * sqrt(n_B * tile_m + n_A * tile_n), u_half = 2^-11
 * (F16) / 2^-8 (BF16), n_B = adds per element of the B-side checksum (MFMA block columns per tile
 * - 1), n_A the same for the A side (two-sided only).  The errors of the B-side sums enter the
 * comparison weighted with the column sums of the A tile, which are at most sqrt(tile_m) times
 * the norms of its columns.  0 for every other scheme and for I8. */
double abft_tolerance_half_coeff(int dtype, int mode, int tile_m, int tile_n);

/* ---- plans: per-layer selection for a network (Sec. 5.3) ------------------- */
typedef struct {
    int32_t M, N, K;
    int32_t dtype;           /* abft_dtype_t */
    int32_t b_layout;        /* abft_blayout_t */
    int32_t has_conv;        /* non-zero: `conv` describes the layer, M and K must match it */
    abft_conv_t conv;
    const void *B;           /* device weights; must stay valid for the life of the plan */
    int64_t ldb;
} abft_layer_t;

typedef struct abft_plan abft_plan_t;

/* Build a plan for `n_layers` layers (host array).  Per layer: picks the scheme
 * (profile = 0: abft_select; profile = 1: times NONE / GLOBAL / THREAD on the device
 * with scratch inputs and keeps the faster protected one, the paper's pre-deployment
 * procedure), computes the offline weight checksum and allocates workspace. */
int abft_plan_create(abft_plan_t **plan, const abft_layer_t *layers, int n_layers, int profile,
                     void *stream);
/* Run layer `layer` of the plan with its chosen scheme on input A (or NHWC x), output C. */
int abft_plan_run(abft_plan_t *plan, int layer, const void *A, int64_t lda, void *C, int64_t ldc,
                  uint32_t *fault_flag, void *stream);
/* Run every layer of the plan in order in one call: A[i], lda[i], C[i], ldc[i] (host arrays of
 * device pointers / leading dimensions) are layer i's input and output.  A layer whose input is
 * the output of the layer before it (A[i] == C[i - 1], lda[i] == ldc[i - 1]) is chained to it and
 * takes its activation checksums from that layer's epilogue where abft_plan_run_chain would.
 * event_layer selects the one layer whose product kernel the abft_set_kernel_events hook brackets
 * (-1: none). */
int abft_plan_run_all(abft_plan_t *plan, const void *const *A, const int64_t *lda, void *const *C,
                      const int64_t *ldc, uint32_t *fault_flag, int event_layer, void *stream);
/* Run `count` consecutive layers of the plan, from layer `first`, as a chain (Sec. 2.4 step 4):
 * layer `first` reads A (lda), every later layer reads the output of the one before it; C[i], ldc[i]
 * (host arrays, i = 0 .. count - 1) are the layers' outputs, each with the layer's activation
 * function applied and its scheme's checks made on the product.
 * When every layer is fully connected in F16 or BF16 with the same batch M, small enough that a
 * launch of its own would run on 32 x 32 tiles, weights in ABFT_B_NK
 * order with 16-byte aligned rows, K a multiple of 64, 16-byte aligned A / C rows, and scheme NONE,
 * GLOBAL or THREAD (and count <= 8), the whole chain runs in ONE kernel launch: the batch is cut into
 * eight slabs of rows, one per die of the GPU, and each die takes its slab through all the layers,
 * the activations staying in that die's L2 (results, checks and flag are those of the per-layer
 * calls).  Otherwise the layers run one launch each, and a layer under ABFT_GLOBAL takes the
 * checksum of its activations from the layer before it instead of forming it (Sec. 2.4 step 4):
 * that layer's epilogue adds up, per column and block of 32 rows, the values it stores (after its
 * activation function, rounded to the output type), which are the column sums of the next layer's
 * input; the next layer multiplies them with its weight checksums, one multiplication per k, and
 * compares as always.  This needs F16 / BF16, the same M, the later layer reading the earlier one's
 * output as a plain M x K matrix (fully connected, or a 1 x 1 convolution of stride 1 without
 * padding) on the direct-to-LDS kernel and the earlier one not on the streaming kernel; a pair
 * of layers that does not qualify runs exactly as under
 * abft_plan_run.  Results are those of
 * abft_plan_run up to the rounding of the checksums (floats here).  Calls on one plan must
 * not overlap (they share the plan's chain state).  The one-launch form never allocates and holds no
 * memset: it can be captured into a HIP graph. */
int abft_plan_run_chain(abft_plan_t *plan, int first, int count, const void *A, int64_t lda,
                        void *const *C, const int64_t *ldc, uint32_t *fault_flag, void *stream);
/* Status word of the plan's chain launches so far (host pointer; synchronises the stream): 0, or
 * bit 0: a wait for a previous layer ran out of its bounded number of polls, bit 1: a workgroup was
 * not placed on the die its index implies.  Either also raised the fault flag of that call and left
 * its outputs incomplete: call abft_plan_chain_reset before the next chain. */
int abft_plan_chain_status(abft_plan_t *plan, uint32_t *status /* host */, void *stream);
/* Clear the chain state (synchronises the stream).  spin_limit: polls one wait may take before it
 * gives up (< 0: the default, about a second); 0 makes every wait that is not already satisfied give
 * up at once, which is how the error path is exercised. */
int abft_plan_chain_reset(abft_plan_t *plan, int spin_limit, void *stream);
/* Diagnostics of a layer's runs through the plan: `report` (device, zero-filled by the caller,
 * or NULL) and `inject` (HOST pointer, copied; NULL: none; testing) are handed to every later run
 * of that layer as abft_gemm takes them.  A chain that holds such a layer runs layer by layer. */
int abft_plan_set_diagnostics(abft_plan_t *plan, int layer, abft_report_t *report /* device */,
                              const abft_fault_t *inject /* host */);
/* How many product launches of this process so far took their activation checksums from the
 * layer before (abft_plan_run_chain, layer by layer); lets a caller see that a chain qualified. */
long long abft_handover_launches(void);
/* Override the scheme of a layer (abft_mode_t; ABFT_AUTO re-applies abft_select). */
int abft_plan_set_mode(abft_plan_t *plan, int layer, int mode);
/* Activation function of a layer (abft_act_t; ABFT_ACT_NONE at creation), fused into the store
 * of C (Sec. 2.4 step 4): every check of the layer sees the accumulators as the product left
 * them, the stored value is the activation of the accumulator, rounded once to the output
 * type.  ABFT_ACT_RELU stores max(x, 0) (a NaN stores 0; a protected scheme has flagged it).
 * With it a chain of layers runs wholly in this library: pass layer l's C as layer l + 1's A
 * to abft_plan_run_all (fp16 / bf16; int8 layers write int32 and do not chain). */
int abft_plan_set_activation(abft_plan_t *plan, int layer, int act);
/* Activation function of a layer (abft_act_t) or a negative error. */
int abft_plan_activation(const abft_plan_t *plan, int layer);
/* Scheme chosen for a layer (abft_mode_t) or a negative error. */
int abft_plan_mode(const abft_plan_t *plan, int layer);
/* Times measured at creation with profile = 1, in microseconds: out[0..2] = NONE, GLOBAL,
 * THREAD (zeros when profile = 0). */
int abft_plan_times(const abft_plan_t *plan, int layer, double *out3 /* host */);
void abft_plan_destroy(abft_plan_t *plan);

/* ---- misc ------------------------------------------------------------------ */
const char *abft_strerror(int code);
/* Library version, e.g. 100 = 1.0.0. */
int abft_version(void);
/* Measurement hook: two hipEvent_t handles (cast to void*) that the following abft_gemm /
 * abft_conv / abft_plan_run calls of the calling host thread record on their stream
 * immediately before and after launching the matrix-product kernel itself (not the
 * checksum pre-pass or the comparison).  NULL, NULL switches it off. */
void abft_set_kernel_events(void *start_event, void *stop_event);
/* Measurement aid behind the choice of MFMA shape for the 256 x 256 tile (no part of the path, no
 * passage of the paper): one launch of a kernel that only multiplies, from registers -- one
 * workgroup of 8 wavefronts per compute unit, each wavefront `iters` times over the 128 x 64 register
 * tile with MFMAs of `shape` x `shape` (32: 32x32x16, 16: 16x16x32; fp16 / bf16, int8 with twice
 * the depth).  `operands` (device) supplies the fragments: at least abft_mfma_probe_bytes() bytes
 * of values of `dtype`; what they hold decides how far the board's power limit lets the clock go.
 * *ops (host) receives the multiply-adds x 2 of the launch.  `sink` (device, 4 bytes) is written
 * only in a case that does not occur (it keeps the work alive).  Errors: ABFT_E_ENUM for an unknown
 * shape or dtype, ABFT_E_NULL, ABFT_E_SHAPE for iters < 1, ABFT_E_HIP. */
size_t abft_mfma_probe_bytes(void);
int abft_mfma_probe(int shape, int dtype, int iters, const void *operands /* device */,
                    float *sink /* device */, double *ops /* host */, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* ABFT_H */
