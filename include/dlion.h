/*
 * dlion.h -- C ABI of the MI355X (gfx950) Distributed Lion optimizer sweep.
 *
 * One iteration of Distributed Lion (Algorithm 1; Section 3.2) for N simulated
 * workers that all live on one GPU:
 *
 *   worker i :  delta_i = sign(beta1*m_i + (1-beta1)*g_i)            (1 bit / coordinate)
 *               m_i    <- beta2*m_i + (1-beta2)*g_i                  (old m_i on the right)
 *   server   :  S = sum_i delta_i ;  Delta = S/N  (averaging)  or  sign(S)  (majority vote)
 *   everyone :  x <- x - lr*(Delta + lambda*x)
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 * Memory.   Every pointer is a DEVICE pointer unless its comment says "host".
 *           The caller owns all memory; the library allocates nothing and keeps
 *           no state between calls other than the launch-shape overrides of
 *           dlion_set_tuning (by default: none) and the address of its static
 *           scratch array per device (dlion_step_noalloc); calls are re-entrant
 *           across streams, except that calls of dlion_step_noalloc share that
 *           array.
 * Streams.  `stream` is a hipStream_t passed as void* (NULL = the default
 *           stream).  Calls only enqueue work and return; they never synchronise.
 * Types.    x and m are fp32.  g is fp32 or bf16 (`g_dtype`); bf16 is widened
 *           to fp32 exactly.  All arithmetic is fp32, every multiply / add /
 *           subtract / divide rounded on its own (no fused multiply-add),
 *           subnormals kept.  (1-beta) is formed once on the host as
 *           `1.0f - beta` in fp32.  Expressions are evaluated exactly as written
 *           above:  c = (beta1*m) + ((1-beta1)*g);  x' = x - (lr*(Delta + (lambda*x))).
 * Workers.  Worker i's momentum is m + i*m_stride, its gradient g + i*g_stride,
 *           its packed update packed + i*packed_stride; strides count ELEMENTS
 *           of the respective type (fp32 / g_dtype / uint64) and must be
 *           >= d (>= W for packed).  Any stride is accepted: bases and strides
 *           need only the alignment of the element type.  Fastest when every row
 *           starts on a 1 KB boundary (m, g strides that are multiples of 256
 *           elements, packed strides that are multiples of 128 words): a wave
 *           then moves whole cache lines that no other wave touches.
 * Sign.     The worker's sign maps 0 (and -0, and NaN) to +1, so that delta is
 *           one bit:  bit = !(c < 0).
 * Packing.  W = ceil(d/64) uint64 words per worker; bit (j % 64) of word (j / 64),
 *           least significant bit first, holds coordinate j: 1 for +1, 0 for -1.
 *           Bits past d in the last word are written as 0.
 * Counts.   p_j = number of workers voting +1 on coordinate j, 0..N, uint16.
 *           The sum of the +-1 votes is S_j = 2*p_j - N.
 * Vote.     Majority vote is sign(S) with sign(0) = 0: a tie leaves only the
 *           weight-decay term.
 * Average.  Delta = (float)S / (float)N, one correctly rounded fp32 division.
 * Errors.   Arguments are validated on the host before anything is enqueued;
 *           on DLION_EINVAL / DLION_EALIGN / DLION_EUNSUPPORTED nothing has been
 *           launched.  DLION_ELAUNCH means the HIP runtime refused a launch (the
 *           status is that launch call's own return value; an error left behind
 *           by an earlier call of the thread is neither reported nor cleared).
 *           A call that enqueues several launches (large d, many workers) may
 *           already have enqueued some of them when a later one is refused:
 *           m is then advanced for some workers / coordinates and not others,
 *           counts, packed and the workspace hold partial results and x may be
 *           updated for some blocks of coordinates only -- the state is not
 *           usable and the step cannot be retried.  No call aborts or throws.
 *           NaN/Inf inputs are not errors: they propagate through the arithmetic.
 * Alignment x, m, g must be aligned to their element size, packed to 8 bytes,
 *           counts to 2 bytes (DLION_EALIGN otherwise).
 * Aliasing. m and x are updated in place; g and packed inputs are read-only;
 *           no two distinct arguments may overlap.
 */
#ifndef DLION_H
#define DLION_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Status, aggregation mode and gradient type travel as plain 32-bit integers, so that a value
 * outside the lists below is an error the library can report (DLION_EINVAL), not undefined
 * behaviour in the caller's or the library's language. */
typedef int32_t dlion_status;
enum {
    DLION_OK = 0,
    DLION_EINVAL = 1,       /* a size, stride, count or enum is out of range, or a pointer is NULL */
    DLION_EALIGN = 2,       /* a pointer is not aligned to its element type */
    DLION_ELAUNCH = 3,      /* the HIP runtime refused a launch (hipLaunchKernel != hipSuccess) */
    DLION_EUNSUPPORTED = 4  /* valid request outside what this build implements */
};

typedef int32_t dlion_mode;  /* Section 3.2, aggregate() */
enum { DLION_VOTE = 0, DLION_AVG = 1 };
typedef int32_t dlion_dtype; /* gradient storage type */
enum { DLION_F32 = 0, DLION_BF16 = 1 };

#define DLION_MAX_WORKERS 65535 /* counts are uint16 */

/*
 * Worker side of one iteration for all N workers (Section 3.2, first display;
 * Algorithm 1, worker-side):  reads m and g, writes m in place and the packed
 * binary updates delta_i -- the d-bit message each worker would send.
 *   m       [N rows of d] fp32, in/out        g      [N rows of d] g_dtype, in
 *   packed  [N rows of W] uint64, out (tail bits zero)
 */
dlion_status dlion_worker_step(float *m, int64_t m_stride, const void *g, int64_t g_stride,
                               dlion_dtype g_dtype, uint64_t *packed, int64_t packed_stride,
                               int64_t d, int32_t N, float beta1, float beta2, void *stream);

/*
 * Server side, the sum (Section 3.2: S_t = sum_i delta_i, held as the count of
 * +1 votes):  counts[j] = sum_i bit_i(j), j < d.
 *   packed  [N rows of W] uint64, in          counts [d] uint16, out
 */
dlion_status dlion_aggregate(const uint64_t *packed, int64_t packed_stride, int64_t d, int32_t N,
                             uint16_t *counts, void *stream);

/*
 * Aggregation and weight update from counts (Section 3.2, second and third
 * displays; Algorithm 1, server-side and the x update):
 *   Delta_j = (2 p_j - N)/N  or  sign(2 p_j - N);   x_j <- x_j - lr*(Delta_j + lambda*x_j).
 *   x [d] fp32, in/out                         counts [d] uint16, in
 */
dlion_status dlion_apply(float *x, const uint16_t *counts, int64_t d, int32_t N, dlion_mode mode,
                         float lr, float lambda, void *stream);

/*
 * Server side and weight update in one pass over the packed streams (Section 3.2,
 * definition of S_t, second and third displays; Algorithm 1, server-side lines and
 * the x update): dlion_aggregate followed by dlion_apply, except that Delta never
 * leaves registers.  counts_or_null, if not NULL, also receives p_j.
 *   x [d] fp32, in/out        packed [N rows of W] uint64, in
 */
dlion_status dlion_aggregate_apply(float *x, const uint64_t *packed, int64_t packed_stride,
                                   int64_t d, int32_t N, dlion_mode mode, float lr, float lambda,
                                   uint16_t *counts_or_null, void *stream);

/*
 * The whole iteration (Algorithm 1, one pass of the loop body; Section 3.2, all three
 * displays): worker step for all N workers, vote count, aggregation and weight update,
 * fused.  Per coordinate it moves m in, m out and g in for each worker and x in and out
 * once.  packed_or_null / counts_or_null, if not NULL, also receive the packed
 * updates and the counts exactly as the unfused calls would write them.
 * Large problems are enqueued as several launches of the same kernel, 67 M coordinates
 * at a time.  With 16 or more workers and d beyond ~16 M the step is faster when each
 * such block is also cut into launches over 8 workers each that hand the votes on (same
 * results bit for bit): in the workspace of dlion_step_ws, else in the counts array
 * (which then holds partial sums until the last launch of a block has run); with
 * neither, each block stays one launch: the library owns no memory.
 */
dlion_status dlion_step(float *x, float *m, int64_t m_stride, const void *g, int64_t g_stride,
                        dlion_dtype g_dtype, int64_t d, int32_t N, dlion_mode mode, float beta1,
                        float beta2, float lr, float lambda, uint64_t *packed_or_null,
                        int64_t packed_stride, uint16_t *counts_or_null, void *stream);

/*
 * dlion_step with a caller-owned workspace (Algorithm 1, the same iteration): same
 * arguments, same results bit for bit.  With 16 or more workers the launches over 8
 * workers each hand the votes on in the workspace (half a byte per coordinate and
 * launch for up to 64 workers, 2 + 2 bytes beyond), a block of coordinates at a time.
 *   workspace_or_null  device memory, 16-byte aligned, at least workspace_bytes long;
 *                      scratch: its contents before and after the call mean nothing.
 *                      Calls that share a workspace must be ordered (same stream).
 *   workspace_bytes    dlion_step_workspace_bytes(d, N) gives the full benefit; less is
 *                      accepted (smaller blocks), and when it holds fewer than 32768
 *                      tiles of 256 coordinates it is ignored: the step then runs as
 *                      it does with NULL / 0.
 * dlion_step_workspace_bytes returns 0 when no workspace would be used (N < 16, small d).
 * Errors: as dlion_step; DLION_EINVAL for a negative size or a size without a pointer,
 * DLION_EALIGN for a workspace that is not 16-byte aligned.
 */
dlion_status dlion_step_ws(float *x, float *m, int64_t m_stride, const void *g, int64_t g_stride,
                           dlion_dtype g_dtype, int64_t d, int32_t N, dlion_mode mode, float beta1,
                           float beta2, float lr, float lambda, uint64_t *packed_or_null,
                           int64_t packed_stride, uint16_t *counts_or_null,
                           void *workspace_or_null, int64_t workspace_bytes, void *stream);

int64_t dlion_step_workspace_bytes(int64_t d, int32_t N);

/*
 * dlion_step for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments and the same results
 * bit for bit as dlion_step_ws; the workspace in which launches over 8 workers each hand
 * their votes on is a static array of DLION_NOALLOC_SCRATCH_BYTES (64 MiB) of device memory
 * inside the library, which every GPU the library runs on holds until the process ends.
 * The call allocates and frees nothing (no hipMalloc / hipFree, no library routine that
 * allocates); its device address is looked up once per device, on the first call made with
 * that device current or by dlion_noalloc_init (call it outside a graph capture; the device
 * that is current must be the stream's).
 *   Limits.  Every (d, N) that dlion_step accepts: the step runs in blocks of coordinates
 *            sized to the scratch (44 M coordinates at 32 workers).  Should a launch plan
 *            ever need more than the scratch holds for its smallest block, the call
 *            returns DLION_EUNSUPPORTED before anything is launched.
 *   Sharing. All calls on one GPU share that GPU's scratch, and nothing in it has to be
 *            cleared between calls (every launch writes what a later one reads).  Calls
 *            that overlap on one GPU (different streams, concurrent graph launches) race:
 *            order them.
 *   Errors.  As dlion_step; DLION_ELAUNCH also when the runtime cannot name the current
 *            device or the scratch's address.
 */
#define DLION_NOALLOC_SCRATCH_BYTES (64u << 20)
dlion_status dlion_noalloc_init(void);
dlion_status dlion_step_noalloc(float *x, float *m, int64_t m_stride, const void *g, int64_t g_stride,
                                dlion_dtype g_dtype, int64_t d, int32_t N, dlion_mode mode,
                                float beta1, float beta2, float lr, float lambda,
                                uint64_t *packed_or_null, int64_t packed_stride,
                                uint16_t *counts_or_null, void *stream);

/* ------------------------------------------------------------------------- *
 * Multi-tensor form: the model is a list of K tensors instead of one flat
 * buffer.  Every tensor is an independent flat problem whose packed bits start
 * on a fresh uint64 word:  tensor k owns words [word_begin_k, word_begin_k +
 * ceil(numel_k/64)) of each worker's packed row and counts
 * [64*word_begin_k, 64*word_begin_k + numel_k) of the counts array, which has
 * 64*W_total entries (entries between a tensor's end and its next word boundary
 * are written as 0 by calls that write counts).
 * ------------------------------------------------------------------------- */
typedef struct dlion_seg {
    float *x;           /* [numel] fp32                                             */
    float *m;           /* worker i at m + i*m_stride                               */
    const void *g;      /* worker i at g + i*g_stride (elements of g_dtype)         */
    int64_t m_stride;
    int64_t g_stride;
    int64_t numel;      /* > 0                                                      */
    int64_t word_begin; /* filled by dlion_mt_layout                                */
    int64_t tile_begin; /* filled by dlion_mt_layout (first wave-tile of the tensor)*/
} dlion_seg;

/*
 * Host-only helper (no passage of the paper: the layout of a tensor list is this
 * library's own; Section 5's models are lists of tensors): fills word_begin /
 * tile_begin of segs_host[0..K) (a HOST array) and returns the total words per
 * worker row and the total tile count.  The caller then copies the table to device
 * memory (K*sizeof(dlion_seg) bytes, 8-byte aligned) and passes both copies to the
 * _mt calls: the host copy is what gets validated, the device copy is what the
 * kernels read.  Errors: DLION_EINVAL (null table, K < 1, a numel <= 0),
 * DLION_EUNSUPPORTED (more than 2^31 - 1 tiles of 256 coordinates).
 */
dlion_status dlion_mt_layout(dlion_seg *segs_host, int32_t K, int64_t *total_words,
                             int64_t *total_tiles);

/*
 * Worker side for a tensor list (Section 3.2, first display; Algorithm 1, worker-side),
 * as dlion_worker_step on every tensor:  packed [N rows of W_total] uint64, out.
 */
dlion_status dlion_worker_step_mt(const dlion_seg *segs_host, const dlion_seg *segs_dev, int32_t K,
                                  dlion_dtype g_dtype, uint64_t *packed, int64_t packed_stride,
                                  int32_t N, float beta1, float beta2, void *stream);

/*
 * Server-side sum for a tensor list (Section 3.2, definition of S_t), as dlion_aggregate.
 * packed: rows as dlion_worker_step_mt writes them (the unused bits of every tensor's last
 * word are zero); counts [64*W_total] uint16, out: the counts of those padding positions
 * come out as 0.  Only numel of each segment is read from the table.
 */
dlion_status dlion_aggregate_mt(const dlion_seg *segs_host, const dlion_seg *segs_dev, int32_t K,
                                const uint64_t *packed, int64_t packed_stride, int32_t N,
                                uint16_t *counts, void *stream);

/*
 * Aggregation and weight update from counts for a tensor list (Section 3.2, second and
 * third displays), as dlion_apply:  counts [64*W_total] uint16, in; every x in/out.
 */
dlion_status dlion_apply_mt(const dlion_seg *segs_host, const dlion_seg *segs_dev, int32_t K,
                            const uint16_t *counts, int32_t N, dlion_mode mode, float lr,
                            float lambda, void *stream);

/*
 * Server side and weight update in one pass for a tensor list (Section 3.2, definition of
 * S_t, second and third displays), as dlion_aggregate_apply.
 */
dlion_status dlion_aggregate_apply_mt(const dlion_seg *segs_host, const dlion_seg *segs_dev,
                                      int32_t K, const uint64_t *packed, int64_t packed_stride,
                                      int32_t N, dlion_mode mode, float lr, float lambda,
                                      uint16_t *counts_or_null, void *stream);

/*
 * The whole iteration for a tensor list (Algorithm 1, one pass of the loop body), as
 * dlion_step / dlion_step_ws: one fused kernel over all tensors.  The workspace form
 * hands the votes of 16 or more workers on exactly as dlion_step_ws does;
 * dlion_step_mt_workspace_bytes takes the total tile count that dlion_mt_layout returned.
 */
dlion_status dlion_step_mt(const dlion_seg *segs_host, const dlion_seg *segs_dev, int32_t K,
                           dlion_dtype g_dtype, int32_t N, dlion_mode mode, float beta1,
                           float beta2, float lr, float lambda, uint64_t *packed_or_null,
                           int64_t packed_stride, uint16_t *counts_or_null, void *stream);

dlion_status dlion_step_mt_ws(const dlion_seg *segs_host, const dlion_seg *segs_dev, int32_t K,
                              dlion_dtype g_dtype, int32_t N, dlion_mode mode, float beta1,
                              float beta2, float lr, float lambda, uint64_t *packed_or_null,
                              int64_t packed_stride, uint16_t *counts_or_null,
                              void *workspace_or_null, int64_t workspace_bytes, void *stream);

int64_t dlion_step_mt_workspace_bytes(int64_t total_tiles, int32_t N);

/* ------------------------------------------------------------------------- *
 * Wider rows around the hot path.
 * ------------------------------------------------------------------------- */

/*
 * Server -> worker message for Delta ("Communication Cost" paragraph; Table 1's
 * Server->Worker column) as bit-planes over the same 64-coordinate words as the
 * workers' messages (bit j%64 of word j/64 = coordinate j, bits past d zero):
 *   DLION_VOTE : plane 0 "plus" = (S > 0); plane 1 "tie" = (S == 0) exists only
 *                for even N.  Delta = plus ? +1 : (tie ? 0 : -1).  d bits for odd
 *                N as in Table 1, 2d bits for even N (the cost of tie -> 0).
 *   DLION_AVG  : plane b = bit b of the count p, b < ceil(log2(N+1)); the
 *                "log(N) d" bits of Table 1.  Delta = (2p - N)/N.
 * dlion_delta_planes: number of planes (host helper; 0 for invalid arguments).
 */
int32_t dlion_delta_planes(int32_t N, dlion_mode mode);

/*
 * Server side in wire format: packed worker messages in, Delta planes out
 * (delta: [planes rows of W] uint64, row stride delta_stride >= W).
 */
dlion_status dlion_aggregate_encode(const uint64_t *packed, int64_t packed_stride, int64_t d, int32_t N,
                                    dlion_mode mode, uint64_t *delta, int64_t delta_stride, void *stream);

/*
 * Worker side of the down-link: decode the planes and take the step
 * x <- x - lr*(Delta + lambda*x) (Section 3.2, third display).
 */
dlion_status dlion_apply_encoded(float *x, const uint64_t *delta, int64_t delta_stride, int64_t d,
                                 int32_t N, dlion_mode mode, float lr, float lambda, void *stream);

/*
 * Worker step / fused step with each worker's own coefficients (footnote of
 * Algorithm 1).  beta1, beta2: DEVICE arrays of N floats; (1 - beta) is formed
 * in fp32 on the device.  beta1[i] == beta2[i] gives the sign-momentum worker
 * of the D-SIGNUM comparison (Section 5).  Everything else as in
 * dlion_worker_step / dlion_step / dlion_step_ws (the workspace is sized by
 * dlion_step_workspace_bytes and used in the same way).
 */
dlion_status dlion_worker_step_pw(float *m, int64_t m_stride, const void *g, int64_t g_stride,
                                  dlion_dtype g_dtype, uint64_t *packed, int64_t packed_stride,
                                  int64_t d, int32_t N, const float *beta1, const float *beta2,
                                  void *stream);
dlion_status dlion_step_pw(float *x, float *m, int64_t m_stride, const void *g, int64_t g_stride,
                           dlion_dtype g_dtype, int64_t d, int32_t N, dlion_mode mode,
                           const float *beta1, const float *beta2, float lr, float lambda,
                           uint64_t *packed_or_null, int64_t packed_stride, uint16_t *counts_or_null,
                           void *stream);
dlion_status dlion_step_pw_ws(float *x, float *m, int64_t m_stride, const void *g, int64_t g_stride,
                              dlion_dtype g_dtype, int64_t d, int32_t N, dlion_mode mode,
                              const float *beta1, const float *beta2, float lr, float lambda,
                              uint64_t *packed_or_null, int64_t packed_stride,
                              uint16_t *counts_or_null, void *workspace_or_null,
                              int64_t workspace_bytes, void *stream);

/*
 * Global Lion, the full-precision comparison scheme (Appendix, "Global Lion
 * Convergence"; the G-Lion baseline of Section 5):
 *   c_i = beta1*m_i + (1-beta1)*g_i;  m_i <- beta2*m_i + (1-beta2)*g_i;
 *   x <- x - lr*(sign(mean_i c_i) + lambda*x).
 * The mean is the fp32 sum over i = 0..N-1 in that order divided by (float)N;
 * the sign maps 0 to +1 as the worker sign does (N = 1 is then the same
 * single-worker Lion).  sign_bits_or_null, if given, receives the W words of
 * sign(mean c) packed like a worker's message, so that agreement with the
 * majority vote can be counted.
 */
dlion_status dlion_global_lion_step(float *x, float *m, int64_t m_stride, const void *g,
                                    int64_t g_stride, dlion_dtype g_dtype, int64_t d, int32_t N,
                                    float beta1, float beta2, float lr, float lambda,
                                    uint64_t *sign_bits_or_null, void *stream);

/*
 * Memory-rate probe for benchmarks (no passage of the paper: it computes nothing of the
 * method).  One-wave workgroups as in the real kernels: wave t reads the t-th 1 KB piece
 * of each of `rows` rows of src (row r at src + r*src_row_stride_bytes), loads_in_flight
 * (1, 2, 4, 8 or 16) rows at a time, folds them with XOR, and, if write != 0, writes one
 * 1 KB piece to dst; with write == 0 nothing is written (dst must still be valid).
 * rows = 1, write = 1 is a plain copy; rows = k gives a k : 1 read : write byte mix.
 * bytes_per_row must be a multiple of 1024, pointers and stride multiples of 16
 * (DLION_EINVAL / DLION_EALIGN otherwise); waves_per_cu caps the resident waves per
 * compute unit (0 = no cap).  It moves rows*bytes_per_row bytes in and
 * (write ? bytes_per_row : 0) bytes out.
 */
dlion_status dlion_membench(const void *src, int64_t src_row_stride_bytes, int32_t rows, void *dst,
                            int64_t bytes_per_row, int32_t write, int32_t loads_in_flight,
                            int32_t waves_per_cu, void *stream);

/* Text for a status code (static storage, never NULL). */
const char *dlion_status_str(dlion_status s);

/* Library version, major*10000 + minor*100 + patch. */
int dlion_version(void);

/* ------------------------------------------------------------------------- *
 * Launch-shape overrides, for tuning runs and for tests that must reach a
 * variant the library would not pick at their sizes.  Nothing here changes a
 * result.  Every field: -1 = the library decides (the default).
 * ------------------------------------------------------------------------- */
typedef struct dlion_tuning {
    int32_t unroll;             /* worker/fused kernels: workers whose loads a wave issues back to back (1, 2, 4, 8) */
    int32_t blocks_per_cu;      /* worker/fused kernels: resident one-wave workgroups per compute unit, 0 = no cap     */
    int32_t pass_workers;       /* workers per launch of a step, 0 = all workers in one launch                        */
    int32_t step_quads;         /* worker/fused kernels: 1 = four consecutive tiles per XCD, 0 = plain numbering      */
    int32_t sliced_waves;       /* bit-sliced server kernels: waves per workgroup (1, 8, 16)                          */
    int32_t sliced_min_workers; /* server side: the per-nibble kernel below this N, the bit-sliced one from it on     */
    int32_t apply_blocks;       /* dlion_apply_encoded: resident workgroups per compute unit, 0 = no cap              */
    int32_t blocks_per_cu_pass; /* as blocks_per_cu, for the launches of a step that only hand their votes on        */
    int64_t block_tiles;        /* worker/fused kernels: tiles (256 coordinates) per launch, 0 = all in one launch    */
    int32_t group_blocks;       /* server side, few-worker kernel: resident 8-wave workgroups per compute unit, 0 = no cap */
    int32_t group_max_workers;  /* server side: the few-worker kernel for every call with N up to this (0 = never, at most 120) */
} dlion_tuning;

/* Fills *t with -1 everywhere. */
void dlion_tuning_defaults(dlion_tuning *t);

/*
 * Installs the overrides for every later call in this process (NULL = back to the
 * defaults).  Host-only, not thread-safe: do not call it while another thread is
 * inside the library.  DLION_EINVAL for a value outside the ranges above.
 */
dlion_status dlion_set_tuning(const dlion_tuning *t);
void dlion_get_tuning(dlion_tuning *t);

#ifdef __cplusplus
}
#endif
#endif /* DLION_H */
