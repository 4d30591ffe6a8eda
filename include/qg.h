/*
 * qg -- group-quantized matrix-vector and small-batch matrix products on MI355X (gfx950).
 *
 * The operation is the one of QIGen (arXiv 2307.03738): a weight matrix is stored as b-bit
 * integer codes q with one scale s and one zero-point z per group of G consecutive inputs,
 * What = s * (q - z) (Section 2, quantization and dequantization, eq. (1)), and the hot path
 * is y = What x computed straight from the packed codes (eq. (2), Algorithm 1), plus its
 * matrix form for a few prompt tokens.
 *
 * Orientation: W is [N][K] row-major, N outputs, K inputs (the paper writes the transpose:
 * its n is K here, its m is N).  Groups run along k.  b is 2, 3 or 4.
 *
 * Conventions for every call
 *   - All data pointers are DEVICE pointers owned by the caller, unless a parameter is
 *     marked HOST.  The library never allocates or frees device memory and never
 *     synchronises: work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and the call returns at once.  Buffers must stay valid until that
 *     work has run.
 *   - Return value: QG_OK (0) or a positive qg_status.  On an error nothing is enqueued and
 *     no output is touched.  No exceptions, no abort.
 *   - Outputs are overwritten, never accumulated into.  Results do not depend on the launch
 *     order of workgroups: there are no floating-point atomics.
 *   - NaN or Inf in W, x or X: unspecified.
 */
#ifndef QG_H
#define QG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    QG_OK = 0,
    QG_ERR_NULL = 1,        /* a required pointer is NULL */
    QG_ERR_SHAPE = 2,       /* N, K, M <= 0; K % G != 0; G not a multiple of the cell size */
    QG_ERR_UNSUPPORTED = 3, /* bits not in {2,3,4}; unknown layout; too many grouped problems */
    QG_ERR_ALIGN = 4,       /* a pointer is not 16-byte aligned */
    QG_ERR_WORKSPACE = 5,   /* workspace missing or smaller than qg_workspace_bytes() */
    QG_ERR_DEVICE = 6       /* the HIP runtime refused the launch */
} qg_status;

typedef enum {
    /* The paper's format (Section 3 "Data format", Algorithm 2): per output n the codes
     * along k form a little-endian bit stream, code k at bits [b*k, b*k+b), cut into 32-bit
     * words; word w of output n at uint32 [w][n] (n contiguous).  A blob in this layout is
     *   uint32 codes [K*b/32][N] | float scales [K/G][N] | uint32 zeros [ceil(K/G*b/32)][N]
     * with the zero-points packed by the same rule along the group index (b bits each,
     * zero-padded to a word).  Needs K*b % 32 == 0. */
    QG_LAYOUT_CANONICAL = 0,
    /* The layout qg_gemv and qg_gemm_small read.  Opaque; a pure permutation of the same
     * codes, scales and zero-points (plus zero padding), fixed by (N, K, bits, group). */
    QG_LAYOUT_DEVICE = 1,
    /* The layout qg_gemv_narrow reads (made from a QG_LAYOUT_DEVICE blob by qg_to_narrow): the same
     * codes, scales and zero-points in records of 16 outputs x 4 steps of K (codes, then their
     * scales, then their zero-points).  Only qg_packed_bytes, qg_to_narrow, qg_from_narrow and the
     * qg_gemv*_narrow calls know it. */
    QG_LAYOUT_DEVICE_NARROW = 2
} qg_layout;

/* Smallest granule of codes the kernels decode at once: 8 codes (one word) at 4 bits, 16
 * (one word) at 2 bits, 32 (three words, Section 3) at 3 bits.  A group must be a whole
 * number of cells: G % qg_cell(bits) == 0. */
int qg_cell(int bits);

const char *qg_status_string(int status);

/* Identifier of the sources and flags this library was built from (a hash the build step
 * passes in); a loader compares it with the sources it sees to refuse a stale library. */
const char *qg_build_id(void);

/* Size in bytes of a packed blob (codes, scales and zero-points) in the given layout;
 * 0 if the shape is not accepted. */
size_t qg_packed_bytes(int64_t N, int64_t K, int bits, int group, int layout);

/* Size in bytes of the scratch buffer qg_gemv (M = 1) or qg_gemm_small (M > 1) needs for
 * this problem (meeting slots of the K-split reduction for the GEMV; partial results of the
 * K split for the GEMM).  For a grouped launch, the sum over its problems.  0 if the shape is
 * not accepted.
 * The buffer must be prepared once before its first use with qg_workspace_init (it fills it
 * with the "empty slot" pattern); every qg_gemv call leaves it prepared again.  A buffer
 * belongs to one problem shape and one of the two entry points, and two calls that overlap
 * in time must not share one. */
size_t qg_workspace_bytes(int64_t N, int64_t K, int bits, int group, int M);
int qg_workspace_init(void *workspace, size_t bytes, void *stream);

/* Per-group min-max round-to-nearest quantization (Section 2; the integer-zero form
 * q = clamp(rint(w/s) + z, 0, 2^b - 1)):
 *   lo = min(0, min w), hi = max(0, max w) over the group
 *   s  = (hi - lo) / (2^b - 1)            fp32 division; s = 1, z = 0 if hi == lo
 *   z  = clamp(rint(-lo / s), 0, 2^b - 1)
 *   q  = clamp(rint(w / s) + z, 0, 2^b - 1)   ties to even, integer addition of z
 * every step one IEEE binary32 operation.
 *   W [N][K] fp32 in;  q [N][K] one code per byte, s [N][K/G] fp32, z [N][K/G] bytes out.
 * Needs K % G == 0 and G % 4 == 0; W and q 16-byte aligned. */
int qg_quantize(const float *W, int64_t N, int64_t K, int bits, int group,
                uint8_t *q, float *s, uint8_t *z, void *stream);

/* Bit-packing of codes, scales and zero-points into one blob of qg_packed_bytes() bytes
 * (Section 3 "Data format").  q, s, z as produced by qg_quantize.  `packed` 16-byte
 * aligned.  Codes and zero-points must be < 2^b (not checked). */
int qg_pack(const uint8_t *q, const float *s, const uint8_t *z, int64_t N, int64_t K,
            int bits, int group, int layout, void *packed, void *stream);

/* Inverse of qg_pack for either layout: returns q, s, z in the qg_quantize arrangement. */
int qg_unpack(const void *packed, int64_t N, int64_t K, int bits, int group, int layout,
              uint8_t *q, float *s, uint8_t *z, void *stream);

/* y[n] = sum_k s[n][k/G] * (q[n][k] - z[n][k/G]) * x[k]   (eq. (2); Algorithm 1)
 * evaluated per group as s * (sum q x - z * sum x) in fp32.  The sums of q x are exact-product
 * sums: on the vector ALU fp32 FMAs; on the matrix cores x goes in without loss of more than
 * fp32 rounding -- as 32-bit fixed point relative to the largest |x| of each run of 128 (4
 * bits) or 256 k (an error of at most 2^-30 of that largest |x| per term, below the rounding
 * of the fp32 sum it enters; the built-in choice), or as three bf16 parts that add up to x.
 * (The fixed point keeps that precision while the largest |x| of a run is at least 2^-97;
 * NaN and infinity in x reach y through the sum of x of their group.)
 *   packed: QG_LAYOUT_DEVICE blob;  x [K] fp32, 64-byte aligned;  y [N] fp32 (overwritten).
 * workspace: qg_workspace_bytes(N, K, bits, group, 1) bytes, 16-byte aligned. */
int qg_gemv(const void *packed, int64_t N, int64_t K, int bits, int group,
            const float *x, float *y, void *workspace, size_t workspace_bytes, void *stream);

/* qg_gemv for callers that cannot allocate device memory or carry a workspace around: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * product, same kernels and the same bits in y as qg_gemv; the meeting slots of the K-split
 * live in a scratch array inside the library (QG_NOALLOC_SCRATCH_BYTES per GPU, held from the
 * library's load until the process ends) instead of a caller's workspace.  The call allocates
 * and frees nothing and enqueues two kernels on `stream`: a fill that puts the slots it may
 * use into their empty state (the array keeps what the last call on that GPU left), then the
 * product.  Problems whose slots do not fit (more than QG_NOALLOC_MAX_N outputs) are refused
 * with QG_ERR_WORKSPACE before anything is enqueued.  All calls on one GPU share that GPU's
 * array: two calls that overlap in time on one GPU (different streams, or two host threads)
 * race and give undefined results; calls on one stream, or otherwise ordered, are safe. */
#define QG_NOALLOC_SCRATCH_BYTES (8u << 20)
#define QG_NOALLOC_MAX_N 63488            /* 992 tiles of 64 outputs x 8448 bytes of slots */
int qg_gemv_noalloc(const void *packed, int64_t N, int64_t K, int bits, int group,
                    const float *x, float *y, void *stream);

/* Several independent products in ONE kernel launch (the seven linear layers of a decoder
 * block at batch 1 are each only microseconds of memory traffic).  `descs` is a HOST array
 * of `count` <= QG_MAX_GROUPED problems; they may differ in shape, bits and group (one
 * launch per distinct (bits, group) pair with groups up to one step of the kernel -- 128
 * codes at 4 bits, 256 at 2 and 3 bits; problems with longer groups, up to one group per
 * output, share one launch per bit width).  Workspace: the sum of qg_workspace_bytes(). */
#define QG_MAX_GROUPED 16
typedef struct qg_gemv_desc {
    const void *packed; /* QG_LAYOUT_DEVICE blob */
    int64_t N, K;
    int bits, group;
    const float *x;     /* [K], 64-byte aligned */
    float *y;           /* [N] */
} qg_gemv_desc;
int qg_gemv_grouped(const qg_gemv_desc *descs /* HOST */, int count,
                    void *workspace, size_t workspace_bytes, void *stream);

/* The gated MLP input of a LLaMA block in one launch: the packed matrix holds two projections
 * of the same x, "gate" in outputs [0, I) and "up" in outputs [I, 2I) (a QG_LAYOUT_DEVICE blob
 * of 2I x K), and
 *   h[n] = silu(y[n]) * y[I + n],   y = What x as in qg_gemv,   silu(t) = t / (1 + exp(-t))
 * The two products are the linear layers of Section 3 "Computation" as they sit side by side
 * in a LLaMA block; the elementwise step that follows them there is folded into the kernel's
 * epilogue.  I must be a multiple of 64.
 *   x [K] fp32, 64-byte aligned;  h [I] fp32 (overwritten);
 * workspace: qg_workspace_bytes(2 I, K, bits, group, 1) bytes, prepared by qg_workspace_init. */
int qg_gemv_swiglu(const void *packed, int64_t I, int64_t K, int bits, int group,
                   const float *x, float *h, void *workspace, size_t workspace_bytes, void *stream);

/* Prompt-phase form for M <= 128 tokens:
 *   Y[m][n] = sum_k X[m][k] * s[n][k/G] * (q[n][k] - z[n][k/G])
 * on the matrix cores (bf16 operands, fp32 accumulation), one of two ways by layout:
 *   - 4-bit codes, G a multiple of 32 that divides or is a multiple of 128, K % 128 == 0: the
 *     weights are dequantized to bf16(s (q - z)) on their way into the matrix instruction, X is
 *     rounded to bf16;
 *   - any width, G a whole number of pairs of cells up to one step (4 bits: 16 ... 128; 2 bits:
 *     32 ... 256; 3 bits: 64 ... 256) or a multiple of a step, K % 16 == 0: the codes enter the
 *     matrix instruction as exact bf16 integers, X is rounded to bf16, and scale and zero-point
 *     are applied in fp32 once per group and element of Y (eq. (2)); X is converted by a
 *     kernel of its own first, so a call enqueues two or three kernels.
 * Where both apply (4 bits) the first is used, except beyond 64 rows on matrices of 4096 tile-steps
 * or more (64 outputs x 128 k each), where the second measured faster; qg_set_gemm_tuning and
 * qg_gemm_autotune choose otherwise.
 * Every other layout (odd numbers of cells per group, K % 16 != 0 only with M == 1) runs
 * qg_gemv once per row in fp32, 16 rows per launch; with K % 16 != 0 and M > 1 the call returns
 * QG_ERR_UNSUPPORTED.  M == 1 is qg_gemv.
 *   X [M][K] fp32 row-major, 64-byte aligned;  Y [M][N] fp32 row-major (overwritten).
 * workspace: qg_workspace_bytes(N, K, bits, group, M) bytes (converted activations and partial
 * results of a K split; for the row-by-row form, qg_gemv's meeting slots, to be prepared with
 * qg_workspace_init). */
int qg_gemm_small(const void *packed, int64_t N, int64_t K, int bits, int group,
                  const float *X, int M, float *Y,
                  void *workspace, size_t workspace_bytes, void *stream);

/* The GEMV on the narrow layout: y = What x as qg_gemv computes it (eq. (1), (2), Algorithm 1;
 * same arithmetic, same <= 1e-4 bound, bitwise deterministic), for launches made of short matrices,
 * where it is faster.  A workgroup covers the whole K of its 16 outputs, so nothing is added
 * across workgroups: these calls need no workspace and allocate nothing.
 * Formats: K a whole number of steps (128 k at 4 bits, 256 at 2 and 3), G from 16 (32 at 3 bits)
 * up to one step and dividing a step, K <= 32768 at 4 bits and 65536 otherwise; anything else
 * returns QG_ERR_UNSUPPORTED (from qg_packed_bytes: 0).
 *   qg_to_narrow:   packed = QG_LAYOUT_DEVICE blob (DEVICE) -> narrow, qg_packed_bytes(...,
 *                   QG_LAYOUT_DEVICE_NARROW) bytes (DEVICE, 16-byte aligned, caller's); the 16-byte
 *                   pieces of codes and the scales move as they are (4 bits: bit 7 of every code byte
 *                   inverted), the zero-points are packed anew, padding is zero; qg_from_narrow is its
 *                   inverse and gives back the QG_LAYOUT_DEVICE blob byte for byte.
 *   qg_gemv_narrow / qg_gemv_grouped_narrow: as qg_gemv / qg_gemv_grouped with `packed` in the
 *                   narrow layout (descs HOST; x 64-byte aligned; y overwritten).
 * qg_last_narrow_kernel: name of the kernel instance of the last such launch ("" before). */
int qg_to_narrow(const void *packed, int64_t N, int64_t K, int bits, int group, void *narrow, void *stream);
int qg_from_narrow(const void *narrow, int64_t N, int64_t K, int bits, int group, void *packed, void *stream);
int qg_gemv_narrow(const void *narrow, int64_t N, int64_t K, int bits, int group,
                   const float *x, float *y, void *stream);
int qg_gemv_grouped_narrow(const qg_gemv_desc *descs /* HOST */, int count, void *stream);
const char *qg_last_narrow_kernel(void);
/* Measurement knob of the narrow GEMV (process-wide): tiles of 16 outputs a wavefront takes against
 * the same staged x, 1 or 2; 0 restores the built-in choice. */
int qg_set_narrow_tuning(int tiles_per_wave);

/* Launch-shape knobs for measurement sweeps (process-wide, not thread-safe; while one of them
 * is non-zero they apply to every launch and the recorded tunings below are not consulted).  0
 * restores the built-in choice.  waves_per_block in 1..16 = most wavefronts that share one tile of 64
 * outputs inside a workgroup; bytes_per_wave = packed code bytes one wavefront streams;
 * kernel = 1: multiply-adds on the vector ALU; 2: on the matrix cores with the 32 x 32 x 16
 * instruction (where that kernel exists: groups of at least two cells and at most one step,
 * and, at 2 and 3 bits, groups of whole steps); 3: with the 4 x 4 x 4 instruction (groups of
 * whole cells up to one step, and, at 2 and 3 bits, groups of whole steps) on bf16; 4: with
 * the 4 x 4 x 4 instruction on int8 (4-bit groups of at least 16 weights). */
int qg_set_gemv_tuning(int waves_per_block, int bytes_per_wave, int kernel);
/* Records a launch shape (same three values) for every later qg_gemv / qg_gemv_grouped /
 * qg_gemv_swiglu / qg_gemv_noalloc launch of this process whose list of (N, K, bits, group) equals
 * that of `descs` (HOST; only the shapes are read, in order) -- what qg_gemv_autotune does with
 * its result, for a caller that has kept such a result from an earlier run (the paper keeps the
 * outcome of its search per matrix size and machine, Section 3).  The table holds 64 lists; a
 * 65th replaces the oldest.  Other launches keep the built-in choice. */
int qg_gemv_record_tuning(const qg_gemv_desc *descs /* HOST */, int count, int waves_per_block,
                          int bytes_per_wave, int kernel);
/* Forgets every recorded tuning (GEMV and small-M GEMM). */
void qg_clear_tuning(void);
/* Name of the kernel instance the last qg_gemv / qg_gemv_grouped / qg_gemv_swiglu launch of this
 * process used (its last launch, if the call made several), e.g. "gemv_mma4i<4, 16>"; "" before
 * the first launch.  HOST string owned by the library.  For benchmark reports. */
const char *qg_last_gemv_kernel(void);
/* Search for the fastest launch shape of one grouped launch -- this machine's counterpart of the
 * paper's parameter search (Section 3, Algorithm 4 with the resource model of eqs. (3)-(5)).
 * `descs` holds `sets` copies of the launch back to back (set i at descs + i * count; same
 * shapes, normally different packed buffers, so that a cache cannot serve the weights; sets = 1
 * times one set again and again).  Each of the 168 candidates (team size x bytes per wavefront x
 * vector-ALU or one of the three matrix-core kernels) is first priced against the machine's
 * budget: registers per lane and LDS per workgroup of its kernel instance bound the wavefronts a
 * compute unit holds, and those times the bytes a wavefront keeps requested must cover the
 * memory system's round trip (8 TB/s x 1.5 us / compute units; for launches too small to get
 * there, half of what the best candidate reaches).  Candidates below that are dropped; the
 * others run the launch `repeats` times, rotating over the sets.  The call WAITS for the GPU
 * (as qg_gemm_autotune does; no other call), records the fastest for launches with this list of
 * shapes as qg_gemv_record_tuning would (the knobs of qg_set_gemv_tuning are left as they were;
 * they have to be 0 for the recorded shape to be used), and reports it (HOST pointers, each may be NULL; best_us = microseconds per launch).  The outputs
 * y are overwritten as by qg_gemv_grouped; all sets share the workspace. */
int qg_gemv_autotune(const qg_gemv_desc *descs /* HOST */, int count, int sets,
                     void *workspace, size_t workspace_bytes, void *stream, int repeats,
                     int *waves_per_block, int *bytes_per_wave, int *kernel, float *best_us);
/* What the last qg_gemv_autotune did: us[c] (HOST, `capacity` >= 168 entries, may be NULL) =
 * microseconds per launch of candidate c, or -1 if the budget dropped it, with
 * c = ((kernel - 1) * 6 + team index) * 7 + size index over teams {0, 2, 4, 8, 12, 16} and
 * bytes per wavefront {0, 4096, 8192, 16384, 32768, 49152, 65536}; and the two counts. */
int qg_gemv_autotune_report(float *us /* HOST */, int capacity, int *timed, int *dropped);

/* Same for qg_gemm_small: splits in 1..8 = number of K ranges handled by different
 * workgroups (clamped to what the shape allows); shape in 1..12 = workgroup shape (how many
 * rows, tiles and K slices the wavefronts of a workgroup cover, and which of the two kernels;
 * ignored if it does not fit M),
 * shape = -1: the kernel for up to 16 rows whatever the number of tiles; shape = 13: the
 * raw-code kernel wherever it takes the layout.
 * 0 restores the built-in choice. */
int qg_set_gemm_tuning(int splits, int shape);
/* The launch-shape search of qg_gemm_small for one problem (N, K, bits, group, M) -- Section 3,
 * Algorithm 4 with the resource model of eqs. (3)-(5), on this machine's terms.  The 120
 * candidates are the 15 values of `shape` above (0, -1, 1..13) x 1..8 K ranges.  Each is planned
 * without being launched and priced: registers per lane and LDS per workgroup of its kernel
 * instance give the workgroups the chip holds at once and so the rounds the launch needs; a round
 * costs a workgroup's fixed time (3.3 us) plus its iterations (2 us each), every further kernel
 * of the call 3 us.  Candidates the planner maps to a plan already seen are skipped, candidates
 * priced above 1.5 times the cheapest are dropped, the others run the product `repeats` times,
 * rotating over the `sets` packed buffers in packed_sets (HOST array of DEVICE pointers, same
 * matrix shape; different buffers keep a cache from serving the weights).  WAITS for the GPU,
 * records the fastest for later qg_gemm_small calls on the same (N, K, bits, group, M) (used
 * while both knobs of qg_set_gemm_tuning are 0; 64 problems are kept; qg_clear_tuning forgets
 * them) and reports it (HOST pointers, each may be NULL).  Y is overwritten as by qg_gemm_small. */
int qg_gemm_autotune(const void *const *packed_sets /* HOST */, int sets, int64_t N, int64_t K,
                     int bits, int group, const float *X, int M, float *Y, void *workspace,
                     size_t workspace_bytes, void *stream, int repeats,
                     int *splits, int *shape, float *best_us);
/* What the last qg_gemm_autotune did: us[c] (HOST, `capacity` >= 120, may be NULL), c = shape
 * index * 8 + (K ranges - 1) with shape index 0 for shape 0, 1 for shape -1 and i + 1 for shape
 * i >= 1: microseconds per call, -1 = dropped by the price, -2 = not a plan of its own (or the layout has no such kernel). */
int qg_gemm_autotune_report(float *us /* HOST */, int capacity, int *timed, int *dropped);

#ifdef __cplusplus
}
#endif
#endif /* QG_H */
