/*
 * shflbw - Shfl-BW (shuffled block-wise) sparse weight x dense activation
 * product for AMD MI355X (gfx950), C ABI.
 *
 * Problem statement (Algorithm 1 of the paper: data A.row_indices,
 * A.metadata, A.values, B[K][N]; result C[M][N]; Section 4.3: both dense
 * matrices are row-major with the batch/token dimension innermost):
 *
 *     Y[M][N] = (W .* mask)[M][K] * X[K][N]
 *
 * where the mask is a Shfl-BW pattern (Section 3.1): after the row
 * permutation `perm`, every group of V consecutive stored rows keeps the
 * same set of columns.  `perm[i]` is the ORIGINAL row of stored row i: stored
 * row i holds W[perm[i]] and its result is written to Y[perm[i]]
 * (reordered write-back, Section 4.2).
 *
 * General rules
 *  - Every function returns an int status: SHFLBW_OK (0) or a negative
 *    shflbw_status.  Nothing aborts or throws across this boundary.  A short
 *    text for the last failure on the calling thread is kept in
 *    shflbw_last_error().
 *  - "host" pointers are ordinary process memory; "device" pointers are HIP
 *    device memory of the current device.  The library never allocates device
 *    memory: the packed matrix lives in a caller-owned device buffer that
 *    must outlive every call using it.
 *  - shflbw_spmm / shflbw_conv2d only enqueue work on the given HIP stream
 *    (a hipStream_t passed as void*; NULL = the default stream) and return
 *    without synchronising.  Launch errors are returned; execution errors
 *    surface at the caller's next synchronisation.  One failure has no HIP
 *    error: a bounded hand-over wait of the shared-slab kernel that ran out
 *    (see shflbw_device_status); it shows as NaN in Y and in that status.
 *  - Y / out are fully overwritten (no accumulate-into).
 *  - Activations and weights are 16-bit floating point, IEEE binary16 or
 *    bfloat16 (one format per packed matrix, chosen at shflbw_compress);
 *    products are accumulated in binary32 on the matrix cores; the result is
 *    rounded once to the requested output type (the operands' format, or
 *    binary32).
 */
#ifndef SHFLBW_H
#define SHFLBW_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct shflbw_matrix shflbw_matrix; /* opaque; owns host copies of the packed arrays */

typedef enum {
    SHFLBW_F16 = 0,  /* IEEE binary16 */
    SHFLBW_BF16 = 1, /* bfloat16 */
    SHFLBW_F32 = 2   /* IEEE binary32 (output only) */
} shflbw_dtype;

typedef enum {
    SHFLBW_NCHW = 0, /* x innermost */
    SHFLBW_CHWN = 1  /* batch innermost: the layout the paper assumes (Section 4.3) */
} shflbw_layout;

typedef enum {
    SHFLBW_OK = 0,
    SHFLBW_ERR_NULL_ARG = -1,      /* a required pointer is NULL */
    SHFLBW_ERR_BAD_SHAPE = -2,     /* M % V != 0, unsupported V, non-positive size, leading dimension too small, ... */
    SHFLBW_ERR_BAD_PERM = -3,      /* perm is not a permutation of 0..M-1 */
    SHFLBW_ERR_BAD_PATTERN = -4,   /* mask differs inside a permuted row group; detail in shflbw_last_error() */
    SHFLBW_ERR_BAD_DTYPE = -5,     /* dtype enum not supported for this argument */
    SHFLBW_ERR_NOT_ON_DEVICE = -6, /* spmm/conv2d before shflbw_bind_device */
    SHFLBW_ERR_HIP = -7,           /* a HIP runtime call failed; text in shflbw_last_error() */
    SHFLBW_ERR_NO_MEMORY = -8,     /* host allocation failed */
    SHFLBW_ERR_BAD_OPTION = -9,    /* unknown tuning value */
    SHFLBW_ERR_HANDOVER = -10      /* a kernel's bounded wait ran out; see shflbw_device_status */
} shflbw_status;

/*
 * Offline step (a) of Section 4.1-4.3 (host only, no GPU needed): check the
 * pattern, reorder the rows into vector-wise form, keep the original row
 * indices, and store the kept V x 1 vectors stitched into V x T_K tiles in
 * the order the matrix cores consume them.
 *
 *  W     host, M x K of wdtype (SHFLBW_F16 or SHFLBW_BF16; 16-bit patterns), row-major,
 *        leading dimension ldw >= K (elements).  The activations given to
 *        shflbw_spmm / shflbw_conv2d later must have the same type.
 *  mask  host, M x K bytes, row-major, leading dimension K; non-zero = kept.
 *        NULL: a V x 1 vector is kept iff any of its V weights is non-zero.
 *        Kept weights whose value is zero are stored like any other.
 *  perm  host, M int32; NULL = identity.
 *  V     rows per group: 16, 32, 64 or 128.  M must be a multiple of V.
 *  out   receives a new handle; release it with shflbw_destroy.
 * Groups may keep different numbers of columns, including none.
 */
int shflbw_compress(const void* W, int ldw, const uint8_t* mask, const int32_t* perm,
                    int M, int K, int V, shflbw_dtype wdtype, shflbw_matrix** out);

/*
 * Pattern search (Section 5), host only: from the weights alone, choose the row shuffle
 * and the kept V x 1 vectors; the results feed shflbw_compress.  Importance = |w|;
 * unstructured pruning to the non-zero ratio beta gives a binary mask; K-Means with
 * clusters of the fixed size V on the rows of that mask groups the rows; vector-wise
 * pruning to the non-zero ratio alpha on the shuffled matrix; the shuffle is undone.
 *  W      host, M x K of wdtype (SHFLBW_F16 or SHFLBW_BF16), finite, leading dimension
 *         ldw >= K.  V must be 16, 32, 64 or 128 and divide M.
 *  alpha  target non-zero ratio in [0, 1]: every group keeps round(alpha*K) vectors.
 *  beta   ratio of the unstructured step; negative = 2*alpha (capped at 1), the value
 *         the paper recommends.
 *  iterations  K-Means rounds at most (it stops when no row moves); 0 = no shuffle,
 *         i.e. plain vector-wise pruning.
 *  perm_out  M int32: perm_out[i] = original row of stored row i.
 *  mask_out  M x K bytes (leading dimension K), original row order; conforms to the
 *         pattern under perm_out.
 * Deterministic: comparisons are exact and ties go to the lower index.
 * Cost: a K-Means round compares every row with every cluster centre, O(M * (M/V) * K)
 * byte operations, and holds 12 bytes per (row, cluster) pair; the unstructured step holds
 * 4 bytes per weight.  Flat indices are 32-bit: M*K or M*(M/V) above 2^32 - 1 is refused
 * with SHFLBW_ERR_BAD_SHAPE.
 */
int shflbw_pattern_search(const void* W, int ldw, int M, int K, int V, double alpha, double beta,
                          int iterations, shflbw_dtype wdtype, int32_t* perm_out, uint8_t* mask_out);

void shflbw_destroy(shflbw_matrix* A);

/* Shape and sparsity of a packed matrix.  Any out pointer may be NULL.
 * nnz counts kept weights (V per kept vector, no padding);
 * sparsity = 1 - nnz / (M*K). */
int shflbw_info(const shflbw_matrix* A, int* M, int* K, int* V, int* groups,
                int64_t* nnz, double* sparsity);

/* Test hooks that expose the logical vector-wise form (host only).
 * shflbw_row_indices: copies the M original-row indices (Section 4.2).
 * shflbw_group_columns: writes the ascending kept columns of group g into
 *   cols[0..cap) and returns their count (>= 0), or a negative status; with
 *   cols == NULL it only returns the count.
 * shflbw_decompress: writes (W .* mask) as M x K binary16 with leading
 *   dimension ldw, original row order; bitwise equal to the masked input. */
int shflbw_row_indices(const shflbw_matrix* A, int32_t* rows_out);
int shflbw_group_columns(const shflbw_matrix* A, int g, int32_t* cols, int cap);
int shflbw_decompress(const shflbw_matrix* A, void* W_out, int ldw);

/* Bytes of device memory the packed matrix needs (multiple of 256). */
size_t shflbw_device_bytes(const shflbw_matrix* A);

/* Copy the packed arrays into dev_buf (device, caller-owned, at least
 * shflbw_device_bytes(A) bytes, 256-byte aligned) on `stream` and remember
 * the address.  The copy is complete when the call returns. */
int shflbw_bind_device(shflbw_matrix* A, void* dev_buf, void* stream);

/* Kernel selection, for measurement.  kernel: 0 = automatic, 1 = per-wave
 * gather kernel, 2 = shared-slab kernel for shflbw_spmm / staged kernel for
 * shflbw_conv2d (the call then fails with SHFLBW_ERR_BAD_OPTION when the
 * matrix, the operands or the shape do not allow it), 3 = gather kernel with
 * the k-steps of a tile split over the wavefronts of a workgroup (the variant
 * for very few output columns; shflbw_conv2d treats 3 like 1).
 * tile_n: 0 = automatic, else the number of output columns one wavefront of
 * the gather kernel owns (64 or 128). */
int shflbw_set_tuning(shflbw_matrix* A, int kernel, int tile_n);

/* The shared-slab kernel hands chunks of X from its loader wavefronts to its
 * compute wavefronts through flags in LDS (Alg. 1's pipeline, without
 * workgroup barriers).  Every wait on a flag is bounded: a wavefront that has
 * polled `tries` times goes on regardless, so a lost hand-over never hangs;
 * it sets a word in the matrix's device buffer, and the failure is visible in
 * the data: every 32 (V) x 128 output tile whose wavefront finished after a
 * wait of its workgroup had run out is stored as NaN, so Y never holds
 * plausible numbers computed from activations that were not there.  (This
 * also holds for shflbw_conv2d where it runs as shflbw_spmm.)
 *
 * shflbw_device_status: waits for `stream`, reads that word back and clears
 *   it.  SHFLBW_OK if no wait ran out in any launch on this matrix since the
 *   last call (or since shflbw_bind_device); SHFLBW_ERR_HANDOVER otherwise:
 *   results of those launches are not to be trusted.  Synchronises the
 *   stream; meant for tests and for a check per batch, not per launch.
 * shflbw_set_wait_limit: polls per wait before a wavefront gives up (default
 *   2^20, about 50 ms).  tries >= 0; 0 makes every wait give up at once, which
 *   is how the tests force the condition (every kernel still ends normally). */
int shflbw_device_status(shflbw_matrix* A, void* stream);
int shflbw_set_wait_limit(shflbw_matrix* A, int tries);

/*
 * Linear layer (Algorithm 1: BulkLoadMeta / StitchTile / WarpMMA loop, then
 * ReorderedWriteBack):  Y = (W .* mask) X.
 *  X  device, K x N of the matrix's wdtype, row-major, leading dimension ldx >= N.
 *  Y  device, M x N of ydtype (the matrix's wdtype, or SHFLBW_F32), leading dimension
 *     ldy >= N.  Must not overlap X.
 * N == 0 is a no-op.  Groups without kept columns produce zero rows.
 * Fast path: N, ldx, ldy multiples of 8 and 16-byte aligned bases; other
 * shapes take a slower element-wise path with the same result.
 */
int shflbw_spmm(const shflbw_matrix* A, const void* X, int64_t ldx, void* Y, int64_t ldy,
                int64_t N, shflbw_dtype ydtype, void* stream);

/*
 * shflbw_spmm for callers that cannot allocate device memory (code that runs where
 * hipMalloc is forbidden or fails: tight serving loops, harnesses that own all device
 * memory): the packed arrays go into a device image that the library itself holds, a
 * static array of SHFLBW_UNBOUND_MAX_BYTES on every GPU it is used on, instead of a
 * caller-owned buffer; no shflbw_bind_device is needed, and a binding the handle may have
 * is neither used nor changed.  Every call copies A's packed arrays (host to device, on
 * `stream`), clears the hand-over status block with a small kernel, and launches exactly
 * what shflbw_spmm launches; X, Y and the result are those of shflbw_spmm, bit for bit.
 * Allocates nothing (no hipMalloc / hipFree).
 *  - A packed matrix larger than SHFLBW_UNBOUND_MAX_BYTES (see shflbw_device_bytes) is
 *    refused with SHFLBW_ERR_BAD_SHAPE.
 *  - All calls on one GPU share the one image, which keeps the last call's contents: calls
 *    whose work can overlap on a GPU (different streams, different threads) race on it and
 *    must be ordered by the caller.  Calls on one stream are ordered by the stream.
 *  - The host arrays of A are read until the copies have been issued; with pageable host
 *    memory the runtime has consumed them when the call returns.
 */
#define SHFLBW_UNBOUND_MAX_BYTES (8u << 20)
int shflbw_spmm_unbound(const shflbw_matrix* A, const void* X, int64_t ldx, void* Y, int64_t ldy,
                        int64_t N, shflbw_dtype ydtype, void* stream);

/*
 * 2-D convolution as implicit GEMM (Section 4.1): the unfolded feature map
 * exists only in on-chip buffers.  A has M = C_out rows and K = C_in*R*S
 * columns flattened as k = (c*R + r)*S + s.  Cross-correlation (no kernel
 * flip), zero padding, dilation 1, groups 1.
 *  in   device, the matrix's wdtype: [batch][C_in][H][W] (NCHW) or [C_in][H][W][batch] (CHWN).
 *  out  device, ydtype (the matrix's wdtype, or SHFLBW_F32): [batch][C_out][H_out][W_out] or [C_out][H_out][W_out][batch],
 *       H_out = (H + 2*pad_h - R)/stride_h + 1, W_out likewise.
 * A workgroup copies the part of the input its output positions can touch into
 * LDS once and gathers from there; inputs with too many channels for that take
 * the per-wave gather kernel.
 * A 1x1 convolution with unit stride and no padding is the linear-layer
 * product itself (CHWN: one matrix; NCHW with H*W a multiple of 4: one per
 * image, all in one launch) and runs as shflbw_spmm does.
 */
int shflbw_conv2d(const shflbw_matrix* A, const void* in, void* out,
                  int batch, int C_in, int H, int W, int R, int S,
                  int stride_h, int stride_w, int pad_h, int pad_w,
                  shflbw_layout layout, shflbw_dtype ydtype, void* stream);

/*
 * LayerNorm-side transposition (Section 4.3, discussion of the activation
 * layout: models whose LayerNorm leaves the features contiguous hand their
 * activations to these kernels through a transposition folded into that
 * LayerNorm).
 *  x      device, N x K of dtype (SHFLBW_F16 or SHFLBW_BF16): N tokens, K features
 *         innermost, leading dimension ldx >= K.
 *  gamma, beta  device, K values of dtype, or NULL (1 and 0).
 *  normalize    non-zero: per token, subtract the mean over the K features, divide by
 *         sqrt(biased variance + eps), multiply by gamma, add beta (statistics in
 *         fp32).  Zero: copy only (gamma, beta, eps ignored).
 *  out    device, K x N of dtype, leading dimension ldo >= N: the matrix shflbw_spmm
 *         takes as X.  Must not overlap x.
 * K, N, ldx, ldo must be multiples of 8 and all bases 16-byte aligned
 * (SHFLBW_ERR_BAD_SHAPE otherwise).  N == 0 is a no-op.  Enqueues on `stream` only.
 */
int shflbw_layernorm_transpose(const void* x, int64_t ldx, const void* gamma, const void* beta,
                               float eps, int normalize, void* out, int64_t ldo, int64_t N,
                               int K, shflbw_dtype dtype, void* stream);

const char* shflbw_status_string(int status);
const char* shflbw_last_error(void); /* thread-local, never NULL */

/* Which kernel the calling thread's most recent successful shflbw_spmm or shflbw_conv2d
 * launched, as "name<template arguments>" (the automatic choice of set_tuning(0, 0) is
 * made per call from the matrix and the operand shape).  Thread-local, never NULL; empty
 * before the first launch. */
const char* shflbw_last_kernel(void);

#ifdef __cplusplus
}
#endif
#endif /* SHFLBW_H */
