/*
 * easyquant.h -- C ABI of the MI355X (gfx950) EasyQuant quantization library.
 *
 * EasyQuant (arXiv 2403.02775) quantizes one weight matrix at a time without any
 * data (Algorithm 1):
 *   1. find the (n sigma) outliers of the weight and keep them verbatim (Eq. 3);
 *   2. for the remaining "normal" values, optimise the quantization range of every
 *      output channel (or group) with Adam, using the gradient of the
 *      reconstruction error ||Q[x] - x||^2 with respect to the range (Eq. 2, Sec. 4.2);
 *   3. quantize the normal values at that range (Eq. 1);
 *   4. dequantize as  Mask * W + (1 - Mask) * Q[W]  (Eq. 4).
 * The output format below follows Sec. 5, Implementation: the quantized normal values
 * plus the position and the original value of every outlier.
 *
 * Conventions that hold for every entry point
 * -------------------------------------------
 *  - Matrices are row-major, ROW = OUTPUT CHANNEL (out_features x in_features), so a
 *    row is what the paper calls a channel sharing one range (Sec. 5, Setup).  A
 *    "unit" is one row (group_size = 0) or group_size consecutive elements of a row.
 *  - Every pointer marked DEVICE is GPU memory owned by the caller; the library
 *    never allocates, frees or retains device memory.  Every pointer marked HOST is
 *    read before the call returns.
 *  - Calls enqueue work on `hip_stream` (a hipStream_t passed as void*, NULL = the
 *    default stream) and return without waiting for it.  eq_quantize_matrix / _batch first
 *    copy their descriptors into the workspace on that stream, in one piece, from a pinned
 *    host block that the library owns and reuses once the copy has completed (a few hundred
 *    KB, allocated on first use): the call does not depend on how the runtime treats
 *    pageable memory and never waits for work queued earlier.
 *  - Return value: EQ_OK or a negative EQ_E_* code for problems visible on the host
 *    (nothing is enqueued then).  Conditions only the GPU can see are reported in
 *    the per-matrix DEVICE status word (EQ_S_* bits), valid once the stream is idle.
 *  - Thread-safe for calls that use distinct outputs and workspaces.
 */
#ifndef EASYQUANT_H_
#define EASYQUANT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* exported symbol (the library is built with hidden visibility by default) */
#define EQ_API __attribute__((visibility("default")))

/* element type of W: outliers keep their original floating-point type (Fig. 1); this library
 * takes the two 16-bit formats. */
enum { EQ_F16 = 0, EQ_BF16 = 1 };
/* EQ_SYMMETRIC is the paper's setting (Sec. 5, Setup).  EQ_ASYMMETRIC is an extension:
 * an integer zero-point fixed from min/max at initialisation, only the range optimised. */
enum { EQ_SYMMETRIC = 0, EQ_ASYMMETRIC = 1 };
/* scope of mean / sigma in Eq. 3: one row (default), one unit, or the whole matrix (Eq. 3 as printed). */
enum { EQ_STAT_ROW = 0, EQ_STAT_GROUP = 1, EQ_STAT_MATRIX = 2 };
/* which iterate of the optimisation is returned: the best of the trajectory (step 0
 * included, so never worse than min/max scaling), or the last one (the ranges of step 100 /
 * 500, as in Sec. 5, Setup). */
enum { EQ_SELECT_BEST = 0, EQ_SELECT_LAST = 1 };

/* return codes */
enum {
  EQ_OK = 0,
  EQ_E_NULL = -1,         /* a required pointer is NULL */
  EQ_E_SHAPE = -2,        /* rows/cols/ld/group_size inconsistent (see eq_quantize_matrix) */
  EQ_E_PARAM = -3,        /* bits, mode, dtype, scope, select or a hyper-parameter out of range */
  EQ_E_ALIGN = -4,        /* W, W_out or x not 16-byte aligned; codes not 16-byte aligned in a quantize
                             call (4-byte in the consumers); another output not aligned to its type */
  EQ_E_WORKSPACE = -5,    /* workspace NULL, misaligned (256 B) or smaller than eq_workspace_bytes() */
  EQ_E_UNSUPPORTED = -6,  /* a row too long for on-chip staging (cols > EQ_MAX_COLS) */
  EQ_E_HIP = -7,          /* a HIP runtime call failed (launch, copy); eq_last_hip_error() has the code */
  EQ_E_SCRATCH = -8       /* eq_quantize_matrix_noalloc: the matrix and its outlier capacity need more
                             scratch memory than the library's built-in EQ_STATIC_SCRATCH_BYTES */
};
/* bits of the DEVICE status word */
enum {
  EQ_S_OUTLIER_OVERFLOW = 1, /* more outliers than out_capacity: out_row_ptr holds the true
                                counts (so the caller can re-size and call again); out_col /
                                out_val are incomplete */
  EQ_S_NONFINITE = 2         /* W holds an Inf or NaN: every output of that matrix is unspecified */
};

#define EQ_MAX_COLS 65536

typedef struct eq_params {
  int32_t dtype;       /* EQ_F16 | EQ_BF16 */
  int32_t bits;        /* 2..8 (the paper evaluates 4) */
  int32_t group_size;  /* 0 = one range per row (the paper's per-channel setting); else a
                          multiple of 32 that divides cols (finer grouping, Sec. 5.1) */
  int32_t mode;        /* EQ_SYMMETRIC | EQ_ASYMMETRIC */
  int32_t stat_scope;  /* EQ_STAT_* */
  float   n_sigma;     /* threshold n of Eq. 3; 2.5..3 in the paper; +inf disables outliers */
  int32_t iters;       /* Adam steps T on the range (100 / 500 in the paper); 0 = outlier-aware RTN */
  float   lr;          /* Adam step size on the range (1e-3 / 1e-4 in the paper) */
  float   beta1, beta2, eps; /* Adam moments in [0, 1) and epsilon > 0 (paper silent: 0.9, 0.999, 1e-8) */
  int32_t select;      /* EQ_SELECT_* */
} eq_params;

/* Quantized form of one rows x cols matrix.  All pointers DEVICE, caller-owned.
 * units_per_row = 1 (group_size 0) or cols / group_size. */
typedef struct eq_qmatrix {
  uint32_t* codes;        /* rows * eq_code_words_per_row(cols, bits) words.  Per row, a
                             little-endian bit stream: the unsigned code of column j sits in
                             bits [bits*j, bits*j+bits) of the row's stream (4-bit: even
                             column in the low nibble); rows are padded to whole words.
                             unsigned code = signed level of Eq. 1 + zero_point; an outlier's
                             slot holds zero_point (level 0). */
  float*    scales;       /* rows * units_per_row: s of Eq. 1 (range / D), binary32 */
  uint8_t*  zero_points;  /* rows * units_per_row: 2^(bits-1)-1 in symmetric mode */
  uint32_t* out_row_ptr;  /* rows + 1: exclusive prefix sum of outliers per row (CSR) */
  uint32_t* out_col;      /* out_capacity: column of each outlier, ascending within a row */
  uint16_t* out_val;      /* out_capacity: the outlier's raw 16-bit pattern (lossless) */
  int64_t   out_capacity; /* entries available in out_col / out_val */
  int32_t*  status;       /* one word, EQ_S_* bits; written by the call (0 = fine) */
} eq_qmatrix;

/* Algorithm 1, "Quantize", for one matrix.
 *   W      DEVICE, rows x cols elements of p->dtype, row stride ld elements (ld >= cols,
 *          ld % 8 == 0, W 16-byte aligned).  Read only.  out->codes must be 16-byte aligned
 *          as well (the kernels store code words 128 bits at a time).
 *   rows   >= 0, cols >= 0 with cols % 8 == 0 (cols % 32 == 0 when group_size != 0) and
 *          cols <= EQ_MAX_COLS.  rows == 0 or cols == 0 enqueues nothing but still
 *          clears status / out_row_ptr.
 *   p      HOST.   out  HOST struct of DEVICE pointers (all non-NULL; out_col / out_val
 *          may be NULL when out_capacity == 0).
 *   workspace  DEVICE scratch, 256-byte aligned, at least eq_workspace_bytes() bytes;
 *          contents are undefined afterwards; must not be shared by calls that overlap.
 * The outlier list comes out sorted by (row, column) whatever the execution order.
 * Same inputs give bit-identical outputs on every run.
 *
 * Which kernel serves a matrix is decided from its shape and p alone (the results do not
 * depend on the choice): group_size 128 with row or matrix statistics and cols <= 32768 runs
 * one unit per lane (without optimisation steps, iters == 0, a load-pipelined variant of it);
 * one range per row with cols a multiple of 128 in 2048..32768 spreads the row over
 * cols / 128 lanes (rows of 11008, 13824, 17920 or 22016 columns with 4-bit codes: in
 * equal pieces over 128 or 256 lanes; with at most 4 bits and iters * (cols - 960) >= 57 * cols
 * (60 to 65 steps for rows of 8192 and longer, 108 for rows of 2048; bf16: 80 in place of 57) the rows
 * are sorted first and every step takes its two sums from the sorted row and its exact prefix
 * sums, which needs up to 2 GiB more workspace, counted by eq_workspace_bytes()); everything
 * else goes to a general kernel (one workgroup per row, one wavefront per unit). */
EQ_API int eq_quantize_matrix(const void* W, int64_t rows, int64_t cols, int64_t ld,
                       const eq_params* p, const eq_qmatrix* out,
                       void* workspace, size_t workspace_bytes, void* hip_stream);

/* The same for n independent matrices in ONE pass over the GPU (weights are independent of one
 * another, Sec. 5, Implementation): W, rows, cols, ld, outs are HOST
 * arrays of length n; all matrices share p.  n == 0 is a no-op. */
EQ_API int eq_quantize_batch(int32_t n, const void* const* W, const int64_t* rows, const int64_t* cols,
                      const int64_t* ld, const eq_params* p, const eq_qmatrix* outs,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/* eq_quantize_matrix for callers that cannot allocate or copy: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments and the same outputs,
 * bit for bit, but there is no workspace argument: the scratch memory (descriptors, work items,
 * Adam's bias-correction table, per-row outlier counts and the staging copy of the outlier
 * list) is a built-in device array of EQ_STATIC_SCRATCH_BYTES that every GPU the library runs
 * on holds until the process ends, and the descriptors are written there by a small kernel
 * from by-value arguments instead of being copied from host memory.  The call allocates and
 * frees nothing on the device and enqueues kernels only.
 *   Limit: eq_workspace_bytes(1, &rows, &cols, &out->out_capacity, p) must not exceed
 *   EQ_STATIC_SCRATCH_BYTES (32 MiB), else EQ_E_SCRATCH (nothing is enqueued).  The need is
 *   about 6 bytes per entry of out_capacity plus 8 bytes per row: a 22016 x 8192 matrix with a
 *   capacity of 2 % of its elements takes 21 MiB, a 4096 x 4096 one with the never-overflowing
 *   capacity of eq_outlier_capacity_bound 11 MiB.  (Rows with one range each are always
 *   optimised element by element here: the records of their sorted form would not fit.)
 *   The device that is current when the call is made must be the one hip_stream belongs to;
 *   the address of that device's array is looked up on the first call per device.
 *   All calls on one GPU share that GPU's array: calls that overlap on one GPU (two streams,
 *   two host threads) race; calls on one stream, or otherwise ordered, are safe, and nothing
 *   needs to be cleared between them. */
#define EQ_STATIC_SCRATCH_BYTES (32u * 1024u * 1024u)
EQ_API int eq_quantize_matrix_noalloc(const void* W, int64_t rows, int64_t cols, int64_t ld,
                               const eq_params* p, const eq_qmatrix* out, void* hip_stream);

/* Algorithm 1, "Dequantize" (Eq. 4): W_out[i][j] = round_to_dtype(scale * (code - zero_point))
 * for normal values, the stored raw pattern for outliers.  W_out DEVICE, rows x cols of
 * p->dtype with row stride ld_out (>= cols, % 8 == 0, 16-byte aligned).  Only dtype, bits
 * and group_size of p are read.  q->status is not touched.  The outlier list must be in the
 * form eq_quantize_* writes it: columns ascending within each row (for a malformed list, with
 * an entry out of order or a column >= cols, it is unspecified which entries of that row are
 * applied; nothing outside W_out is ever written).  q->out_col / q->out_val NULL: no outliers.
 * One kernel launch on hip_stream, every argument passed by value, no device memory
 * allocated or copied: the call (like eq_dequant_matvec) may be recorded into a HIP graph;
 * the eq_quantize_* calls may not, they upload descriptors from host memory. */
EQ_API int eq_dequantize(const eq_qmatrix* q, int64_t rows, int64_t cols, const eq_params* p,
                  void* W_out, int64_t ld_out, void* hip_stream);

/* Eq. 4 fused with a matrix-vector product (the serving-time use of a quantized weight, the
 * scenario of the paper's latency paragraph in Sec. 5 for one token): y = W^ x, where W^ is
 * exactly what eq_dequantize would write (every element rounded to p->dtype, outliers verbatim),
 * but W^ never reaches memory: bits/8 bytes are read per weight instead of 2.
 *   x  DEVICE, cols elements of p->dtype, 16-byte aligned.    y  DEVICE, rows binary32 values.
 * Products and sums are binary32 in an unspecified order: y agrees with the exact product to
 * within 3e-5 * sum_j |W^_ij x_j| per row.  q as for eq_dequantize.  cols == 0 gives y = 0.
 * 4-bit codes with one range per row, or with groups of a power of two >= 64 elements, are
 * served from small tables of the 16 values a weight of the row / group can take (the weights
 * are the same bits as with the plain arithmetic that serves every other format). */
EQ_API int eq_dequant_matvec(const eq_qmatrix* q, int64_t rows, int64_t cols, const eq_params* p,
                      const void* x, float* y, void* hip_stream);

/* Bytes of workspace eq_quantize_batch needs for these shapes (HOST arrays of length n);
 * eq_quantize_matrix is the n == 1 case.  0 on invalid arguments. */
EQ_API size_t eq_workspace_bytes(int32_t n, const int64_t* rows, const int64_t* cols,
                          const int64_t* out_capacity, const eq_params* p);

/* Words per row of the packed code stream: ceil(cols * bits / 32). */
EQ_API int64_t eq_code_words_per_row(int64_t cols, int32_t bits);

/* An out_capacity that can never overflow: by Chebyshev's inequality at most 1/n^2 of a
 * statistic scope lies n sigma from its mean (Eq. 3), so rows*cols/n^2 rounded up per row
 * (rows*cols when n <= 1).  Typical weights need 0.3-1 % (Tables 8-9). */
EQ_API int64_t eq_outlier_capacity_bound(int64_t rows, int64_t cols, float n_sigma);

/* Fills *p with the paper's BLOOM setting: 4 bits, per-channel, symmetric, n = 3,
 * Adam lr 1e-3 for 100 steps (Sec. 5, Setup), fp16, row statistics, best iterate. */
EQ_API void eq_default_params(eq_params* p);

/* INSTRUMENTATION for benchmarks (not needed to use the library; off by default, and the
 * quantization and its results are the same with it on).  While enabled, every launch of a main quantization kernel
 * (the kernels that run Algorithm 1's "Quantize"; not the small reset / prefix-sum / gather
 * kernels around them) is bracketed by HIP events on the call's stream.
 * eq_profile_read waits for those events, returns the summed kernel time in milliseconds and
 * the number of launches since the last read, and forgets them.  The list of events is shared by
 * all host threads of the process (a lock guards it): a read returns every thread's launches. */
EQ_API int eq_profile_enable(int on);
EQ_API int eq_profile_read(double* kernel_ms, int32_t* launches);

/* Static description of a return code. */
EQ_API const char* eq_strerror(int code);
/* hipError_t of the most recent EQ_E_HIP on this thread (0 if none). */
EQ_API int eq_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* EASYQUANT_H_ */
