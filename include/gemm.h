/*
 * gemm.h -- C ABI of the MI355X (gfx950) dense matrix-multiplication library.
 *
 * The operation is the paper's MatMul specification (Section 3.1,
 * "Specifications"): three matrices in global memory, each with a shape, an
 * element type and a storage layout,
 *
 *      A : M x K        B : K x N        C : M x N
 *      C(i,j) = sum_{k=0..K-1} A(i,k) * B(k,j)
 *
 * C is OVERWRITTEN (Section 3.2, "Epilog": the accumulator is zero-filled and
 * then stored); there is no alpha/beta and no accumulate-into-C.
 *
 * Pointers
 *   Every matrix pointer is a DEVICE pointer owned by the caller.  The library
 *   neither frees nor retains them.  C must not overlap A or B.
 *
 * Layout and leading dimension
 *   layout is GEMM_ROW_MAJOR or GEMM_COL_MAJOR, given per operand.  Element
 *   (r,c) of a row-major matrix is at index r*ld + c, of a column-major matrix
 *   at r + c*ld (indices in elements).  ld == 0 means packed (row-major: number
 *   of columns, column-major: number of rows); otherwise ld must be at least
 *   that value.  Elements between the packed extent and ld are never written.
 *   Those of A and B may be read (nothing past an operand's last element is),
 *   but their values, NaN included, never influence C.  Pointers need only
 *   element alignment.  Bases and leading dimensions that are multiples of 4
 *   bytes (always the case for binary32) take the direct-load kernels, multiples
 *   of 16 bytes make them fastest; 16-bit operands that are only 2-byte aligned
 *   take slower kernels that stage loads through registers.
 *
 * Element types
 *   gemm_f32    : binary32 operands, IEEE binary32 multiply-add, binary32 C.
 *   gemm_f16f32 : binary16 operands (passed as their 16-bit patterns), products
 *                 accumulated in binary32, binary32 C.
 *   gemm_f16f16 : the same, with C rounded to binary16 at the store.
 *   gemm_bf16f32: bfloat16 operands (16-bit patterns: the upper half of the
 *                 binary32 number of the same value), binary32 accumulation and C.
 *   The order in which the K products are added is unspecified.  Subnormal
 *   operands and results are kept (nothing is flushed to zero); NaN and
 *   infinity propagate through the elements of A and B only.
 *
 * Execution
 *   Work is enqueued on hip_stream (a hipStream_t cast to void*; NULL is the
 *   default stream) of the current device.  The call does not synchronise with
 *   the host, on any path.  Shapes that are split along K keep their partial
 *   sums in a workspace that belongs to the (device, stream) pair: calls on
 *   different streams never share one, calls on one stream are ordered by the
 *   stream, and host threads that share a stream are serialised by the library
 *   for the duration of the launches.  A workspace that is too small is
 *   replaced by a larger one with hipMalloc (the old one is kept until
 *   gemm_shutdown(), since earlier work may still use it), so such a call can
 *   be recorded into a HIP graph only once its stream's workspace has reached
 *   the size it needs, e.g. after the same call was made once outside the
 *   capture; calls that use no K-slices only launch kernels and can always be
 *   captured.  gemm_f16f32_noalloc never allocates.
 *
 * Sizes
 *   M, N, K >= 0 and each below 2^31 - 256.  M == 0 or N == 0: nothing is
 *   done.  K == 0: C is filled with zeros (empty sum).
 *
 * Errors
 *   Functions return GEMM_OK (0) or a negative gemm_status_t; they never abort
 *   or throw.  Nothing is enqueued when a negative value is returned from
 *   argument validation.
 */
#ifndef MI355X_GEMM_H
#define MI355X_GEMM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { GEMM_ROW_MAJOR = 0, GEMM_COL_MAJOR = 1 } gemm_layout_t;

typedef enum {
    GEMM_OK = 0,
    GEMM_ERR_INVALID_ARG = -1, /* negative size, bad layout, small ld, null pointer */
    GEMM_ERR_HIP = -2,         /* a HIP runtime call or the kernel launch failed */
    GEMM_ERR_UNSUPPORTED = -3, /* size beyond the stated limits, unknown forced config */
    GEMM_ERR_WORKSPACE = -4    /* the split-K workspace could not be allocated */
} gemm_status_t;

/* C = A*B, binary32 throughout (paper Section 3.1, MatMul with float elements). */
int gemm_f32(int64_t M, int64_t N, int64_t K,
             const float *A, int layoutA, int64_t lda,
             const float *B, int layoutB, int64_t ldb,
             float *C, int layoutC, int64_t ldc,
             void *hip_stream);

/*
 * C = A*B, binary16 operands, binary32 accumulation and result (the mixed
 * precision of the paper's Tensor Core kernels, Section 4.2, with the
 * accumulator kept in binary32).
 */
int gemm_f16f32(int64_t M, int64_t N, int64_t K,
                const uint16_t *A, int layoutA, int64_t lda,
                const uint16_t *B, int layoutB, int64_t ldb,
                float *C, int layoutC, int64_t ldc,
                void *hip_stream);

/*
 * C = A*B, binary16 operands, binary32 accumulation, binary16 result: the
 * operand types of the paper's executable tensor-core spec (Section 4.2,
 * "Supporting HMMA", where C is FP16 as well) and of the half-precision library
 * routine it is measured against (Section 5.3).  Each element of C is the
 * binary32 sum rounded once to binary16, to nearest even; sums beyond the
 * binary16 range become infinities.  C is passed as 16-bit patterns.
 */
int gemm_f16f16(int64_t M, int64_t N, int64_t K,
                const uint16_t *A, int layoutA, int64_t lda,
                const uint16_t *B, int layoutB, int64_t ldb,
                uint16_t *C, int layoutC, int64_t ldc,
                void *hip_stream);

/*
 * C = A*B, bfloat16 operands, binary32 accumulation and result: the same MatMul
 * specification (Section 3.1) on the matrix instruction of Section 4.2 with the
 * target's other 16-bit operand format (1 sign, 8 exponent, 7 fraction bits).
 * Products of two bfloat16 numbers are exact in binary32; the sum is rounded as
 * in gemm_f16f32.  Arguments, layouts and errors as for gemm_f16f32.
 */
int gemm_bf16f32(int64_t M, int64_t N, int64_t K,
                 const uint16_t *A, int layoutA, int64_t lda,
                 const uint16_t *B, int layoutB, int64_t ldb,
                 float *C, int layoutC, int64_t ldc,
                 void *hip_stream);

/*
 * gemm_f16f32 for callers that cannot allocate device memory: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * operation, arguments, layouts and errors as gemm_f16f32, but the call never
 * calls hipMalloc or hipFree: the partial sums of a shape that is split along K
 * go to a fixed array of GEMM_NOALLOC_SCRATCH_BYTES that every GPU the library
 * runs on holds until the process ends.  The automatic selection only picks
 * K-slice counts whose partials (slices * M * N' * 4 bytes, N' = N rounded up
 * to a multiple of 32) fit the array; a
 * forced configuration that needs more is refused with GEMM_ERR_WORKSPACE and
 * nothing is enqueued.  All calls on one GPU share that GPU's array (its
 * contents are whatever the last call left; every call overwrites what it
 * reads), so calls that overlap in time on one GPU -- different streams, or
 * graphs replayed concurrently -- race: order them.
 */
#define GEMM_NOALLOC_SCRATCH_BYTES (64u << 20)
int gemm_f16f32_noalloc(int64_t M, int64_t N, int64_t K,
                        const uint16_t *A, int layoutA, int64_t lda,
                        const uint16_t *B, int layoutB, int64_t ldb,
                        float *C, int layoutC, int64_t ldc,
                        void *hip_stream);

/*
 * Kernel-configuration control (the paper tunes the block tile per input size,
 * Section 5.3; here a heuristic picks it and this hook overrides it).
 * name is "auto" / NULL for the heuristic, or "<tile>[:s<slices>][:safe][:direct|:staged][:regload]" with
 * <tile> a configuration name or "auto", e.g. "t256x256", "t128x128:s4",
 * "auto:s2:safe".  A slice count beyond the number of K slabs means one slab
 * per slice.  ":safe" runs the same kernels with every hand-over of a
 * shared-memory buffer preceded by a wait for all outstanding memory operations
 * and a full barrier (the paper notes, Section 4.1, that removing
 * synchronisation can introduce races: this is the variant to compare against
 * when one is suspected).  ":direct" stores C straight from the accumulator
 * registers (the path edge tiles always take), ":staged" stages whole rows of
 * every interior tile through shared memory (Section 3.2, "Epilog") wherever
 * the rows of C start on 16-byte boundaries; without either the library picks
 * by shape.  ":regload" runs the register-staged kernels whatever the
 * alignment.  Returns GEMM_ERR_UNSUPPORTED for an unknown name.
 * The setting is process-wide.
 */
int gemm_force_config(const char *name);

/*
 * Re-calibration of the selection's cost model (Section 5.3 tunes per input
 * size by measurement; the model's constants were measured on one part):
 * multiplies one term by factor (> 0; 1 = as measured).  term < 0 resets all.
 * Process-wide; GEMM_ERR_INVALID_ARG for an unknown term or factor <= 0.
 */
enum {
    GEMM_COST_SLAB = 0,  /* time a workgroup needs per K slab */
    GEMM_COST_HBM = 1,   /* sustained HBM rate (larger = faster memory) */
    GEMM_COST_L2 = 2,    /* sustained L2-to-CU rate */
    GEMM_COST_FIXED = 3, /* launch, pipeline fill and reduce-pass latencies */
    GEMM_COST_TERMS = 4
};
int gemm_cost_model_scale(int term, double factor);

/*
 * Per-size tuning by measurement (Section 5.3 searches the configurations exhaustively for each
 * input size and keeps the fastest; the cost model above replaces that search at call time, this
 * call performs it).  kind names the entry point (GEMM_KIND_*), the other arguments are that entry
 * point's: the call computes C = A * B like it, then runs the product again with each candidate
 * (tile, K slices) pair -- the max_candidates cheapest by the cost model, or every pair the library
 * has if max_candidates is 0 (9 tiles x up to 6 slice counts; 10-50 ms for a mid-size shape, 1.3 s at 8192^3) --
 * timing each with events on hip_stream (two untimed and six timed launches per pair behind 40 untimed ones, all
 * enqueued back to back; then the four fastest and the cost model's own pick again, twice in turn with 24 timed
 * launches each, the better take of each kept), records the fastest in a process-wide table, computes C
 * once more with it and writes "<tile>:s<slices>" into buf.  Later calls with the same M, N, K,
 * operand width (16-bit or binary32), layouts and alignment class on a device with as many CUs use
 * the recorded pair (so do gemm_query_config*); a forced configuration still overrides it, and
 * gemm_f16f32_noalloc ignores an entry whose partial sums do not fit its array.  The call blocks the
 * host until hip_stream has drained, allocates (events, K-slice workspace), and cannot be captured into a
 * HIP graph.  Errors as the entry point's, plus GEMM_ERR_INVALID_ARG for an unknown kind, a negative
 * max_candidates or no buffer, and GEMM_ERR_HIP if no candidate could be timed.  An empty product
 * (M, N or K zero) records nothing and writes "none".  gemm_tune_clear forgets every recorded pair.
 */
enum {
    GEMM_KIND_F32 = 0,     /* gemm_f32 */
    GEMM_KIND_F16F32 = 1,  /* gemm_f16f32 */
    GEMM_KIND_F16F16 = 2,  /* gemm_f16f16 */
    GEMM_KIND_BF16F32 = 3  /* gemm_bf16f32 */
};
int gemm_tune(int kind, int64_t M, int64_t N, int64_t K, const void *A, int layoutA, int64_t lda, const void *B, int layoutB,
              int64_t ldb, void *C, int layoutC, int64_t ldc, void *hip_stream, int max_candidates, char *buf, int buflen);
int gemm_tune_clear(void);

/*
 * The recorded pairs as a text file, so that a service tunes once and later processes start with the picks:
 * gemm_tune_save writes every pair gemm_tune has recorded (one line each: bytes per operand element, M, N,
 * K, alignment class, number of K-contiguous operands, CU count, whether the operands are whole slabs and
 * granules, tile name, K slices; '#' starts a comment line); gemm_tune_load adds the pairs of such a file to
 * the table, replacing entries for the same class.  Host only.  GEMM_ERR_INVALID_ARG if the file cannot be
 * opened or written, or (load) if any line does not parse, names a tile this build does not have or one
 * that cannot serve the line's class, or a K-slice count outside 1 .. 32 (what gemm_tune records): then
 * nothing of the file is taken over.
 */
int gemm_tune_save(const char *path);
int gemm_tune_load(const char *path);

/*
 * The configuration the selection would pick (or the forced one), without touching the
 * device: elem_bytes is 2 (16-bit operands) or 4 (binary32); aligned is the alignment in
 * bytes that the bases and leading dimensions of A and B share: 16 or more (or 1, "yes")
 * means the direct-load kernels at their best, 8 or 4 the direct-load kernels on rows that
 * straddle cache lines, 2 the register-staged kernels on operands whose 16-byte loads the
 * memory pipeline has to split, 0 ("no") the register-staged kernels for another reason (a
 * leading dimension too long for 32-bit tile offsets, a forced ":regload").  Writes "<tile>:s<splits>"
 * into buf (NUL-terminated, truncated to buflen).
 * This is the host side of the per-size tuning of Section 5.3, exposed so that it can be
 * tested without a GPU.
 */
int gemm_query_config(int elem_bytes, int64_t M, int64_t N, int64_t K, int aligned, char *buf, int buflen);

/*
 * gemm_query_config for given layouts of A (M x K) and B (K x N), GEMM_ROW_MAJOR or
 * GEMM_COL_MAJOR each (gemm_query_config assumes both row-major): operands that are not 16-byte
 * aligned cost more or less depending on which of them have K as their contiguous dimension, so
 * the pick can differ.  GEMM_ERR_INVALID_ARG for any other layout value.
 */
int gemm_query_config_layouts(int elem_bytes, int64_t M, int64_t N, int64_t K, int aligned, int layoutA, int layoutB,
                              char *buf, int buflen);

/*
 * Profiling aid (the paper times whole kernels, Section 5; this shows where inside a
 * launch the time goes).  With a device buffer of 8 * workgroups 64-bit words set, the first
 * thread of every workgroup of the following gemm_* launches records a constant-rate 100 MHz
 * clock at the phase boundaries of its tile: word 0 start, 1 first operands landed (direct-load
 * kernels only), 2 K loop done, 3 shared memory free for the epilogue, 4 stores issued,
 * 5 stores complete; word 7 says where it ran (XCC id in the upper half, the hardware id
 * register in the lower).  Workgroups numbered beyond the buffer record nothing; a later
 * launch overwrites an earlier one's records.  NULL switches it off (the default).  The
 * caller owns the buffer and keeps it alive while set.  Process-wide.
 */
int gemm_set_phase_trace(void *device_buffer, int64_t workgroups);

/* Number of tile configurations, and the name of the i-th (NULL if out of range). */
int gemm_num_configs(void);
const char *gemm_config_name(int i);

/*
 * Description of the configuration the last successful call on this thread
 * used, e.g. "f16 t256x256 NT aligned s1".  The string is thread-local storage
 * owned by the library, valid until the thread's next gemm call.
 */
const char *gemm_last_config(void);

/* Text for a status code (static storage). */
const char *gemm_status_string(int status);

/*
 * Frees every K-slice workspace (waits for the work that still uses them).  Safe to call
 * more than once.  A HIP graph that recorded a K-sliced call holds its workspace's address:
 * such a graph must not be replayed after this call.
 */
int gemm_shutdown(void);

#ifdef __cplusplus
}
#endif
#endif /* MI355X_GEMM_H */
