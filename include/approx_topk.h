/*
 * approx_topk.h - C ABI of the MI355X (gfx950) bucketed approximate top-k library.
 *
 * Method: arxiv 2412.04358, Section 2 ("Algorithm design choices"):
 *   Stage 1  split each row of n elements into b interleaved buckets (element i goes to
 *            bucket i mod b, Appendix A.1), keep the k_b largest of every bucket and
 *            concatenate the b*k_b survivors;
 *   Stage 2  if b*k_b > k, keep the k largest of the survivors (an exact top-k).
 *
 * Conventions fixed by this library where the paper is silent:
 *   - "larger" means: greater value, and among equal values the lower column index
 *     (at every stage).  Values compare as IEEE numbers (+0 == -0); rows must not
 *     contain NaN (behaviour is then unspecified, but memory-safe).
 *   - Output order.  Without Stage 2 (b*k_b == k): bucket-major, slot j*k_b + t holds
 *     the t-th largest element of bucket j.  With Stage 2, and for exact_topk: largest
 *     first.
 *   - out_vals carries the selected element's own bits (the sign of a zero survives).
 *
 * All data pointers are DEVICE pointers on the current HIP device.  The caller owns every
 * buffer; the library keeps no pointer after the call's work has finished.  Calls are
 * asynchronous on `stream` (a hipStream_t passed as void*, NULL = the default stream):
 * they enqueue kernels and return; buffers must stay valid until the stream has drained.
 * A per-device scratch pool (partial results, tickets, radix-select state) is owned by
 * the library; it grows on demand (growing allocates, which may synchronise the device)
 * and is shared by all calls on a device.  A call that needs the pool on another stream than
 * the call before it first waits, on the host, for that earlier stream to drain (calls
 * that stay on one stream never wait); calls from different host threads are serialised by
 * a lock around the pool, not around the launches, so threads that share a device should
 * share a stream or order their calls themselves.  Because of the allocation and the wait,
 * approx_topk and exact_topk are not for streams under graph capture: approx_topk_noalloc is.
 *
 * Every function returns ATK_OK (0) or a negative error code.  Arguments are checked on
 * the host before any HIP call is made; nothing is launched when a check fails.
 */
#ifndef APPROX_TOPK_H
#define APPROX_TOPK_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* element types of x / out_vals */
enum { ATK_F32 = 0, ATK_BF16 = 1 };

/* bucket assignment functions of Appendix A.1 */
enum {
    ATK_INTERLEAVED = 0, /* element i goes to bucket i mod b: what the paper uses in all experiments */
    ATK_CONTIGUOUS = 1   /* element i goes to bucket floor(b*i/n): runs of n/b adjacent elements */
};

/* return codes */
enum {
    ATK_OK = 0,
    ATK_ERR_NULL_PTR = -1,    /* a required pointer is NULL */
    ATK_ERR_BAD_SHAPE = -2,   /* m, n or k out of range (m,n,k >= 1, k <= n, n < 2^31, m*n and m*k < 2^40) */
    ATK_ERR_BAD_PARAMS = -3,  /* b, k_b violate 1 <= b <= n, 1 <= k_b <= min(k, n/b), b*k_b >= k */
    ATK_ERR_UNSUPPORTED = -4, /* legal for the method, not implemented here (see each function) */
    ATK_ERR_DTYPE = -5,       /* dtype is neither ATK_F32 nor ATK_BF16 */
    ATK_ERR_HIP = -6,         /* a HIP runtime call failed; see atk_last_hip_error() */
    ATK_ERR_ALIGN = -7,       /* a pointer is not aligned to its element size */
    ATK_ERR_WORKSPACE = -8    /* approx_topk_noalloc: the call needs more scratch than its fixed array holds */
};

/* Largest supported k_b (per-lane insertion buffers live in registers). */
#define ATK_MAX_KB 16

/*
 * Bucketed approximate top-k of every row (Section 2, Stage 1 + Stage 2; Figure 2 left).
 *
 *   x         device, m x n row-major contiguous, element type `dtype`; read only.
 *   m, n      rows, row length.            k   outputs per row, 1 <= k <= n.
 *   b, k_b    buckets per row and survivors per bucket: 1 <= b <= n,
 *             1 <= k_b <= min(k, n/b), b*k_b >= k.
 *   out_vals  device, m x k, element type `dtype`.
 *   out_idx   device, m x k int32 column indices (0-based, within the row).
 *
 * n need not be a multiple of b: bucket j holds the indices j, j+b, ... below n (the short
 * buckets of Figure 2); k_b <= floor(n/b) keeps every bucket long enough.
 *
 * Stage 2 runs inside the same kernel launch as long as its b*k_b candidates fit one workgroup
 * (atk_stage2_max_candidates()); with more, Stage 1 leaves the candidates in library scratch and
 * the long-row exact selection picks the k largest of them in further launches.
 *
 * ATK_ERR_UNSUPPORTED: k_b > ATK_MAX_KB.
 */
int approx_topk(const void *x, int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b, int dtype,
                void *out_vals, int32_t *out_idx, void *stream);

/*
 * The same with the bucket assignment as an argument (Appendix A.1, "Bucket assignment"):
 * ATK_INTERLEAVED is approx_topk itself; ATK_CONTIGUOUS makes bucket j the run of elements
 * ceil(j*n/b) <= i < ceil((j+1)*n/b) (lengths floor(n/b) or ceil(n/b)).  Output order, ties and
 * errors as for approx_topk; any other `assignment` is ATK_ERR_BAD_PARAMS.  Contiguous buckets
 * lose recall on sequences whose neighbours are correlated (the appendix's simulation); they
 * are here to reproduce that comparison.
 */
int approx_topk_assign(const void *x, int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b, int dtype,
                       int assignment, void *out_vals, int32_t *out_idx, void *stream);

/*
 * approx_topk for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, results and errors as approx_topk, but the
 * scratch of plans whose workgroups hand partial lists over (few rows of long rows; Stage 2 over rows split
 * between workgroups) is a fixed array of ATK_NOALLOC_SCRATCH_BYTES inside the library's code object, one
 * per device, held until the process ends: the call allocates and frees nothing, and never synchronises.
 *   - ATK_ERR_WORKSPACE when the plan needs more than the array holds (atk_workspace_bytes() tells:
 *     at most ATK_NOALLOC_STATE_BYTES of tickets and the rest of the array in lists), ATK_ERR_UNSUPPORTED
 *     when Stage 2 would run over more than atk_stage2_max_candidates() candidates.  Nothing is launched then.
 *   - The array keeps the last call's contents; the call clears the tickets it uses with a small fill
 *     kernel before its own launch (one more launch when the plan uses scratch, none otherwise).
 *   - Every call on a device shares that device's array: calls that may overlap on one device (different
 *     streams) race, and must be serialised by the caller.  approx_topk uses other memory and may overlap.
 */
#define ATK_NOALLOC_STATE_BYTES (256 * 1024)
#define ATK_NOALLOC_SCRATCH_BYTES (16 * 1024 * 1024 + ATK_NOALLOC_STATE_BYTES)
int approx_topk_noalloc(const void *x, int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b, int dtype,
                        void *out_vals, int32_t *out_idx, void *stream);

/*
 * Exact top-k of every row, the comparison point (Section 1; the radix-select listing of
 * Appendix D.2 is the algorithm family): the k largest elements, largest first.
 * Arguments as for approx_topk.
 */
int exact_topk(const void *x, int64_t m, int64_t n, int64_t k, int dtype, void *out_vals, int32_t *out_idx,
               void *stream);

/* Static, never-freed description of a return code. */
const char *atk_strerror(int code);

/* hipError_t value of the most recent ATK_ERR_HIP on the calling thread (0 if none). */
int atk_last_hip_error(void);

/* Host-only argument checks (the same ones approx_topk / exact_topk run first). Pointers are not examined. */
int atk_check_approx(int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b, int dtype);
int atk_check_exact(int64_t m, int64_t n, int64_t k, int dtype);

/* Largest b*k_b for which Stage 2 runs on-chip in the same launch (more candidates take further launches). */
int64_t atk_stage2_max_candidates(void);

/* Bytes of library scratch an approx_topk / approx_topk_assign / exact_topk call with these arguments uses
 * (0 if none, <0 = error code). */
int64_t atk_workspace_bytes(int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b, int dtype);
int64_t atk_workspace_bytes_assign(int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b, int dtype, int assignment);
int64_t atk_exact_workspace_bytes(int64_t m, int64_t n, int64_t k, int dtype);
/* The two parts of exact_topk's scratch, which live in separate pools: *state_bytes (words every kernel leaves
 * zeroed: histograms, tickets) and *data_bytes (row states, survivors, copy-out buffers).  Each covers every
 * block of rows the call is run in.  Returns ATK_OK or an error code. */
int atk_exact_workspace_parts(int64_t m, int64_t n, int64_t k, int dtype, int64_t *state_bytes, int64_t *data_bytes);

/*
 * Writes a one-line, human-readable description of the launch plan the library would use
 * (threads per workgroup, lanes per bucket column, row splits, fused Stage 2, ...) into
 * buf (NUL-terminated, truncated to buflen).  Host only; used by tests and the benchmark log.
 * The plan can be overridden for tuning and tests with the environment variable ATK_PLAN (read once, when
 * the library is loaded) or with atk_set_plan_override(), a comma
 * separated list of: T=<threads per workgroup: 64..1024>, S=<workgroups a row is split over>,
 * V=<columns per lane: 1, 2, 4, 8>, P=<lanes of a workgroup sharing a column group: a power of two up to 64>,
 * PK=0 (bf16: no packed queue words), XS=0 / XS=1 (exact_topk with k <= 512: never / also on small
 * inputs guess the threshold from a sample of the row first), XC=<elements of a row per workgroup of
 * exact_topk's sweeps: a power of two from 1024 to 16384>, LN=0 (k_b = 1: the general kernel instead of the
 * one specialised for running maxima), LM=0 (k_b = 1: the lanes of a column merge through per-part lists and
 * a pass over them instead of atomic maxima in LDS), HF=0 / HF=1 (never / whenever the shape allows, two
 * workgroups - a helper and a finisher - share a row of a Stage-2 plan), HQ=<sixty-fourths of the matrix rows
 * that the helper takes: 1..63>, HT=<threads of such a workgroup>, SL=<lanes of a workgroup that stream>,
 * MH=0 / MH=<h> (k_b = 1: split rows never / with h helpers run as helpers and a finisher that meet through
 * mailboxes instead of partial lists and a ticket; HF=0 switches these off as well), BO=0 (Stage 2's bins take their
 * key range from the merged candidates, never from the bounds that come with the merge), RF=0 / RF=<n> (queues of
 * eight slots never / from n load batches on pool their floors).
 * Values the kernels cannot take are ignored or clamped; results never depend on the plan.
 */
int atk_plan_describe(int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b, int dtype, char *buf,
                      int64_t buflen);
/* The same for approx_topk_assign (for ATK_CONTIGUOUS: lanes per bucket Gs, workgroups across the buckets, splits). */
int atk_plan_describe_assign(int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b, int dtype, int assignment,
                             char *buf, int64_t buflen);
/* Replaces the plan override by `spec` (the syntax of ATK_PLAN; NULL or "" = no override).  Host only, process
 * wide, not synchronised with calls running on other threads: meant for sweeps and tests.  Returns ATK_OK. */
int atk_set_plan_override(const char *spec);

/*
 * Choosing (b, k_b) (Section 3 and Appendices C-E).  Host only, no HIP call.
 *
 * atk_expected_recall: Eq. 1 of Appendix C, the expected fraction of the true top-k that the
 *   method returns when top-k positions fall into buckets uniformly (a lower bound on the
 *   recall once k_b is not small against n/b, as the remark after Eq. 1 says).  -1 for
 *   arguments outside 1 <= k_b <= k <= b*k_b.
 * atk_worst_case_recall: Eq. 2 of Appendix C, the recall when the true top-k sit in as few buckets as they can
 *   (floor(b*k/n) buckets full of them and one more with the rest): the lower end of what any input can give, which
 *   the paper calls too pessimistic for real data and leaves out of its discussion.  Stated for b dividing n; -1 for
 *   other arguments or ones Section 2 does not allow.
 * atk_estimate_us: microseconds one approx_topk call with these arguments is expected to take on
 *   an MI355X, in the shape of Appendix D's cost composition (Stage 1 + Stage 2 if b*k_b > k) with
 *   terms fitted to this library's measured timings.  -1 if the arguments are not accepted.
 * atk_advise: among k_b in {1,2,4,8,16} and b*k_b/k in {1,2,4,...,64} that approx_topk accepts,
 *   the pair with the lowest estimate whose Eq. 1 recall is at least min_recall (0 < min_recall <= 1).
 *   Writes *b, *k_b and, when not NULL, *recall and *us.  Returns ATK_OK, or
 *   ATK_ADVISE_BELOW_TARGET (1) when no accepted pair reaches min_recall (then the pair with the
 *   highest recall is written), or an error code.
 */
#define ATK_ADVISE_BELOW_TARGET 1
double atk_expected_recall(int64_t k, int64_t b, int64_t k_b);
double atk_worst_case_recall(int64_t n, int64_t k, int64_t b, int64_t k_b);
double atk_estimate_us(int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b, int dtype);
int atk_advise(int64_t m, int64_t n, int64_t k, int dtype, double min_recall, int64_t *b, int64_t *k_b,
               double *recall, double *us);

/*
 * Measurement utilities (Appendix B.1 protocol, and the roofline's empirical ceiling).
 *
 * atk_read_ceiling: a read-only streaming kernel over `bytes` bytes (multiple of 16, 16-byte
 *   aligned) of device memory at x; every wave xors what it read into its own word of
 *   `sink`, a device buffer of ATK_CEILING_SINK_BYTES bytes.  Contiguous slabs, eight 16-byte
 *   loads per lane in flight, two workgroups of 256 lanes per CU (the fastest of the shapes
 *   tried from 32 MB to 512 MB): the reference for what one pass over x costs on this machine.
 * atk_copy: a plain device-to-device copy kernel of `bytes` bytes (multiple of 16, both pointers
 *   16-byte aligned, buffers must not overlap).  Its read and write volumes are known exactly,
 *   which is what hardware traffic counters are scaled against.
 * atk_sleep: a kernel that spins for about `microseconds` (one wave), used to queue work
 *   behind it so that host launch latency stays out of event timings.
 * atk_trace_approx: approx_topk (same arguments and results) run by a measurement build of the fused kernel in
 *   which lane 0 of every wavefront stores the device's 100 MHz wall clock at the phase boundaries of the
 *   call: trace[(workgroup * ATK_TRACE_WAVES + wavefront) * ATK_TRACE_PHASES + phase], 64-bit words, 0 where a
 *   wavefront never passed.  Phases: 0 start, 1 own share of the row read, 2 own lists merged and handed on,
 *   10 last ticket drawn, 11 other workgroups' lists merged, 3 Stage 2 begins, 4 key range known, 5 histogram,
 *   6 prefix sums, 7 possible winners filed by bin, 8 outputs written, 9 end; words 12 and 13 hold the
 *   wavefront's HW_ID and XCC_ID hardware registers (which CU of which XCD it ran on).  The caller zero-fills `trace`
 *   (device, atk_trace_bytes() bytes for these arguments).  Only the k_b = 1 kernels with 16-byte loads
 *   (b a multiple of 4 in f32, of 8 in bf16) and a fused Stage 2 have this build: ATK_ERR_UNSUPPORTED /
 *   ATK_ERR_HIP otherwise.  The timestamps cost a few stores per wavefront; timings of approx_topk itself
 *   are taken without them.
 */
#define ATK_CEILING_SINK_BYTES 65536
#define ATK_TRACE_WAVES 16
#define ATK_TRACE_PHASES 16
int64_t atk_trace_bytes(int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b, int dtype);
int atk_trace_approx(const void *x, int64_t m, int64_t n, int64_t k, int64_t b, int64_t k_b, int dtype, void *out_vals,
                     int32_t *out_idx, void *trace, int64_t trace_bytes, void *stream);
int atk_read_ceiling(const void *x, int64_t bytes, void *sink, void *stream);
int atk_copy(void *dst, const void *src, int64_t bytes, void *stream);
int atk_sleep(int64_t microseconds, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* APPROX_TOPK_H */
