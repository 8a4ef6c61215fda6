/*
 * nms.h - C ABI of the MI355X (gfx950) data-parallel non-maximum suppression library.
 *
 * The library computes what the paper's two kernels compute ("Proposed Parallel
 * Algorithm": Algorithm 1, the all-pairs map kernel, and Algorithm 2, the row-AND
 * reduce kernel; "Algorithm Correctness": their postconditions):
 *
 *   box i survives  <=>  there is no box j that outranks i with overlap(i, j) >= theta
 *
 *   outranks:  score_j > score_i, or score_j == score_i and j < i        (total order;
 *              the paper's guard is the strict score test of Algorithm 1, the index
 *              tie-break is this library's addition)
 *   overlap:   iw = max(0, (min(x2_i, x2_j) - max(x1_i, x1_j)) + 1)
 *              ih = max(0, (min(y2_i, y2_j) - max(y1_i, y1_j)) + 1)
 *              overlap(i, j) = (iw * ih) / (((x2_j - x1_j) + 1) * ((y2_j - y1_j) + 1))
 *              i.e. intersection over the area of the OUTRANKING box, pixel-inclusive
 *              "+1" (Algorithm 1; MapKernel postcondition).  float32, every operation
 *              rounded to nearest-even on its own, in the order written.
 *
 * An eliminated box still eliminates others (ReduceKernel postcondition: V_i is the
 * AND of the whole row of B).  This is not the sequential greedy procedure.
 *
 * Conventions for every entry point
 *   - Pointers are DEVICE pointers unless a parameter says "host".  `stream` is a
 *     hipStream_t passed as void* (NULL = the default stream).
 *   - Calls only enqueue kernels on `stream` and return; they never allocate device
 *     memory, never synchronise, issue no memset or copy, and keep no state (except
 *     nms_init's pool, below), so they may be captured in a HIP graph.
 *   - The caller owns every buffer.  Buffers must stay valid until the stream has
 *     passed the call.  Inputs are never written.
 *   - Return value: NMS_OK or a negative nms_status.  Arguments are validated on the
 *     host before anything is launched; on error nothing has been enqueued.
 *     n == 0 (or frames == 0) is NMS_OK and enqueues nothing.
 *   - Preconditions that are NOT checked (results unspecified, memory-safe anyway):
 *     coordinates finite with |x| <= 2^40, x2 >= x1, y2 >= y1, scores not NaN.
 *   - Same inputs give the same bits, on any stream.
 *   - A box table ("sorted5") for n boxes is 5 * nms_padded_n(n) floats:
 *     first nms_padded_n(n) rows of (x1, y1, x2, y2) in rank order, then
 *     nms_padded_n(n) areas in rank order.  Rows at or beyond n hold the box (0,0,0,0), area 1.
 *   - An elimination mask for n boxes is nms_mask_words(n) 64-bit words laid out
 *     mask[w * nms_padded_n(n) + r]: bit b of that word is 1 iff the box of rank
 *     64*w + b eliminates the box of rank r.  Only words with w <= r / 64 are written
 *     (the ranked lower triangle; a box is only ever eliminated by a better-ranked
 *     one); bits at or above the diagonal and rows at or beyond n are written as 0.
 *   - Batched calls process `frames` independent frames.  Frame f uses
 *     boxes + f*n_max*4, scores + f*n_max, order + f*n_max, keep_out + f*n_max,
 *     sorted5 + f*5*nms_padded_n(n_max), mask + f*nms_mask_words(n_max).
 *     counts[f] (device, may be NULL = every frame holds n_max boxes) is clamped to
 *     [0, n_max]; keep_out entries at or beyond counts[f] are written 0.
 */
#ifndef NMS_MI355X_H
#define NMS_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define NMS_VERSION 100          /* major*10000 + minor*100 + patch */
#define NMS_TILE 64              /* boxes per tile = wavefront width */
#define NMS_MAX_N 65536          /* largest n (and n_max) accepted */
#define NMS_MAX_FRAMES 65535     /* largest batch accepted */
#define NMS_MAX_MAP_WORKGROUPS 16777215  /* frames (rounded up to 8) x ceil(work units of a frame / 4) must not exceed this:
                                            the pair-test step of a batch is one launch.  A frame of n boxes has about
                                            (n/64)^2 / 8 work units; the limit only binds above some 5,600 boxes per frame
                                            (about 8,000 frames of 16,384 boxes, 500 of 65,536) */
#define NMS_SORT_CHUNK 4096      /* boxes ranked by one workgroup in LDS */
#define NMS_MAX_MATRIX 16384     /* largest capacity of the byte-matrix form (256 MiB of B) */
#define NMS_STATIC_SCRATCH_BYTES 4194304  /* scratch that the library itself holds on every GPU it is loaded on (4 MiB),
                                             used by nms_run_static_batched only */

typedef enum {
    NMS_OK = 0,
    NMS_ERR_INVALID_ARG = -1,   /* null pointer, negative size, NaN threshold */
    NMS_ERR_TOO_LARGE = -2,     /* n > NMS_MAX_N, frames > NMS_MAX_FRAMES, or the batch exceeds NMS_MAX_MAP_WORKGROUPS */
    NMS_ERR_WORKSPACE = -3,     /* workspace missing, misaligned or too small; nms_run without nms_init */
    NMS_ERR_LAUNCH = -4         /* the HIP runtime refused a launch */
} nms_status;

/* Static, never freed.  Unknown codes give "unknown status". */
const char *nms_status_string(int status);
int nms_version(void);
/* HIP runtime's description of the calling thread's most recent NMS_ERR_LAUNCH (static string). */
const char *nms_last_launch_error(void);

/* Host-only size helpers (pure functions; 0 on invalid arguments). */
int nms_padded_n(int n);                                  /* n rounded up to a multiple of NMS_TILE */
size_t nms_mask_words(int n);                             /* ceil(n/64) * nms_padded_n(n) */
size_t nms_sort_workspace_bytes(int n_max, int frames);   /* scratch of nms_sort*: 0 when n_max <= NMS_SORT_CHUNK */
size_t nms_workspace_bytes(int n_max, int frames);        /* scratch of nms_run_ws / nms_run_batched */
/* Which kernels nms_run_batched launches for a batch shape: one of NMS_ROUTE_*; -1 on invalid sizes. */
#define NMS_ROUTE_DIRECT 0
#define NMS_ROUTE_ALL_PAIRS 1
#define NMS_ROUTE_TWO_LAUNCH 2
#define NMS_ROUTE_EARLY_EXIT 3
#define NMS_ROUTE_SMALL_FRAMES 4
int nms_route(int n_max, int frames);

/*
 * Step 1 - rank.  The total order that Algorithm 1 evaluates per pair as
 * "D[i].s < D[j].s", hoisted out of the pair loop so that only the ranked lower
 * triangle of B has to be evaluated.
 *   boxes   [n][4] (x1, y1, x2, y2)      in
 *   scores  [n]                           in
 *   order   [n] int32                     out: order[r] = input index of the box of rank r
 *   sorted5 5 * nms_padded_n(n) floats    out: box table (see above); area as in
 *                                              Algorithm 1's first assignment, per axis
 *   workspace  >= nms_sort_workspace_bytes(n, 1) bytes, 256-byte aligned; may be NULL when that is 0
 */
int nms_sort(const float *boxes, const float *scores, int n,
             int32_t *order, float *sorted5, void *workspace, size_t ws_bytes, void *stream);
int nms_sort_batched(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                     int32_t *order, float *sorted5, void *workspace, size_t ws_bytes, void *stream);

/*
 * Step 2 - map.  Algorithm 1 on the ranked lower triangle, bit-packed and with the
 * polarity inverted (bit = 1 where the paper's B_ij is false).  One 64-bit word per
 * box per 64-box tile of outranking boxes.
 *   sorted5   box table from step 1      in
 *   threshold theta, any float but NaN (no clamping: theta <= 0 eliminates everything
 *             below the top rank, theta > 1 nothing)
 *   mask      nms_mask_words(n) words     out (layout above)
 */
int nms_overlap_mask(const float *sorted5, int n, float threshold, uint64_t *mask, void *stream);
int nms_overlap_mask_batched(const float *sorted5, const int32_t *counts, int n_max, int frames,
                             float threshold, uint64_t *mask, void *stream);

/*
 * Step 3 - reduce.  Algorithm 2's result (V_i = AND of row i of B), i.e. rank r
 * survives iff all its mask words are zero, scattered back to input order
 * (Equation 2 applies V to D index by index).
 *   keep_out [n] bytes, 1 = survives, 0 = eliminated
 */
int nms_reduce(const uint64_t *mask, const int32_t *order, int n, uint8_t *keep_out, void *stream);
int nms_reduce_batched(const uint64_t *mask, const int32_t *order, const int32_t *counts, int n_max, int frames,
                       uint8_t *keep_out, void *stream);

/*
 * The whole path in one call.  No mask is written to memory: the row AND is folded
 * into the pair tests, and the result is the same keep vector as steps 1-3 give.
 * The call picks its route by size (nms_route() names it); every route returns the same bits:
 *   NMS_ROUTE_DIRECT      small work (up to about 2^25 pair slots = frames * n_max^2): one launch.
 *   NMS_ROUTE_SMALL_FRAMES  batches of ten or more frames of 513 to 1024 boxes (of 128 or more
 *                         frames from 449 boxes on), and 2 to about 40
 *                         frames of 1025 to 4096 boxes (which batch sizes depends on the frame
 *                         length; nms_route() tells): one launch without a sort, every victim
 *                         against the two best-ranked of every sixteen input boxes, then the
 *                         victims still alive against the whole frame; rank order enters as a
 *                         compare of the two boxes' (score, index) keys.
 *   NMS_ROUTE_ALL_PAIRS   rank step, then every pair test of the ranked triangle.
 *   NMS_ROUTE_TWO_LAUNCH  frames beyond NMS_SORT_CHUNK boxes, 2^27 <= pair slots < 2^31: rank step,
 *                         every victim against the best 2048 ranks, then only the victims still
 *                         alive against the rest.
 *   NMS_ROUTE_EARLY_EXIT  large batches (frames of 1025 to NMS_SORT_CHUNK boxes from 2^28 pair
 *                         slots, larger frames from 2^31): nms_run_early_exit_batched below.
 * All but DIRECT and ALL_PAIRS skip pair tests of victims that already have an eliminator, so
 * their running time depends on the data.  Callers that want every pair evaluated whatever the
 * size (a fixed running time) call nms_run_ranked_batched.
 *   workspace >= nms_workspace_bytes(n or n_max, 1 or frames) bytes, 256-byte aligned
 *             (always required, whichever route is taken).
 * Two calls that share a workspace must be ordered on one stream.
 */
int nms_run_ws(const float *boxes, const float *scores, int n, float threshold,
               uint8_t *keep_out, void *workspace, size_t ws_bytes, void *stream);
int nms_run_batched(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                    float threshold, uint8_t *keep_out, void *workspace, size_t ws_bytes, void *stream);

/*
 * The two all-pairs routes that nms_run_batched chooses between, callable on their own.
 *   ranked  rank step, then pair tests on the ranked lower triangle (each pair once).
 *           Needs the workspace.  Chosen for batches and large frames.
 *   direct  one launch, no workspace: Algorithm 1 on the full n x n grid of the unsorted
 *           input with the score guard evaluated per pair, row AND finished in the
 *           workgroup.  About 2.5x the arithmetic, so it is chosen only where launch
 *           latency dominates (n_max <= 4096 and frames * n_max^2 up to about 2^25).
 * Both give the same keep_out as nms_run_batched, bit for bit, for any sizes.
 */
int nms_run_ranked_batched(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                           float threshold, uint8_t *keep_out, void *workspace, size_t ws_bytes, void *stream);
int nms_run_direct_batched(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                           float threshold, uint8_t *keep_out, void *stream);

/*
 * The classic sequential greedy rule as a selectable reduce: rank r survives iff no
 * SURVIVING better-ranked box eliminates it (the procedure the paper's introduction and
 * related-work section describe; Algorithms 1 and 2 themselves let eliminated boxes
 * eliminate too).  Same mask, same overlap measure, same tie rule; every box kept by
 * nms_reduce is also kept here.
 *   nms_reduce_greedy*        step 3 alternative on the mask of step 2
 *   nms_run_greedy_batched    rank + map + greedy sweep; needs the mask in its workspace:
 *                             >= nms_greedy_workspace_bytes(n_max, frames) bytes, 256-byte aligned.
 *                             Batches of frames of at most NMS_SORT_CHUNK boxes with
 *                             frames * n_max >= 32 * 4096 take the route below instead (same
 *                             result, bit for bit).
 *   nms_run_greedy_fused_batched   rank, then one workgroup per frame walks the frame in rank
 *                             order, 64 rows a round, and tests only rows that are still alive
 *                             against boxes that survived; the rows left are packed together
 *                             after 2, 4, 8 ... rounds.  No mask, and most of the pair grid is
 *                             never evaluated.  n_max <= NMS_SORT_CHUNK (else NMS_ERR_TOO_LARGE);
 *                             workspace >= nms_workspace_bytes(n_max, frames).  A frame is one
 *                             compute unit's work, so it pays from a few dozen frames on.
 */
int nms_reduce_greedy(const uint64_t *mask, const int32_t *order, int n, uint8_t *keep_out, void *stream);
int nms_reduce_greedy_batched(const uint64_t *mask, const int32_t *order, const int32_t *counts, int n_max,
                              int frames, uint8_t *keep_out, void *stream);
size_t nms_greedy_workspace_bytes(int n_max, int frames);   /* host-only, pure; 0 on invalid arguments */
int nms_run_greedy_batched(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                           float threshold, uint8_t *keep_out, void *workspace, size_t ws_bytes, void *stream);
int nms_run_greedy_fused_batched(const float *boxes, const float *scores, const int32_t *counts, int n_max,
                                 int frames, float threshold, uint8_t *keep_out, void *workspace, size_t ws_bytes,
                                 void *stream);

/*
 * Selectable variants of the rule (the paper's closing section: the map/reduce pattern
 * carries over to the members of the greedy NMS family with changes in the merging step).
 * Every switch at its first value is the default path above.
 *   rule     NMS_RULE_PAPER   every outranking box counts (Algorithms 1 + 2)
 *            NMS_RULE_GREEDY  only outranking boxes that survive themselves count
 *   measure  NMS_MEASURE_OUTRANKING_AREA  intersection / area of the outranking box (Algorithm 1)
 *            NMS_MEASURE_IOU              intersection / ((area_i + area_j) - intersection)
 *   compare  NMS_COMPARE_GE   overlap >= theta eliminates (Algorithm 1: B = overlap < theta)
 *            NMS_COMPARE_GT   only overlap > theta eliminates
 *   ties     NMS_TIES_BY_INDEX  equal scores: the lower index outranks
 *            NMS_TIES_IGNORE    equal scores never eliminate each other (Algorithm 1's strict "<" as printed)
 *   pixel_offset  added to every extent before areas and intersections are formed:
 *            1.0f (the paper's pixel-inclusive convention) or 0.0f (continuous coordinates;
 *            then x2 > x1 and y2 > y1 is an unchecked precondition).  Other values: NMS_ERR_INVALID_ARG.
 *   classes  NULL, or device int32 [frames][n_max]: only boxes with equal labels interact.
 * float32, one rounding per operation, in the order written above; the division is IEEE.
 * nms_run_ex_batched: rank, then the map step with the options; the paper's rule has its row
 * reduction folded into that kernel, the greedy rule takes the sweep on a mask (workspace) or,
 * on large batches, the mask-free walk.  With every option at its default the call is
 * nms_run_batched / nms_run_greedy_batched.
 *   options    HOST pointer, read before the call returns; NULL = all defaults
 *   workspace  >= nms_ex_workspace_bytes(n_max, frames) bytes, 256-byte aligned
 */
enum { NMS_RULE_PAPER = 0, NMS_RULE_GREEDY = 1 };
enum { NMS_MEASURE_OUTRANKING_AREA = 0, NMS_MEASURE_IOU = 1 };
enum { NMS_COMPARE_GE = 0, NMS_COMPARE_GT = 1 };
enum { NMS_TIES_BY_INDEX = 0, NMS_TIES_IGNORE = 1 };
typedef struct nms_options {
    int32_t rule;
    int32_t measure;
    int32_t compare;
    int32_t ties;
    float pixel_offset;
    int32_t reserved;          /* must be 0 */
    const int32_t *classes;    /* device, or NULL */
} nms_options;
size_t nms_ex_workspace_bytes(int n_max, int frames);   /* host-only, pure; 0 on invalid arguments */
int nms_run_ex_batched(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                       float threshold, const nms_options *options, uint8_t *keep_out,
                       void *workspace, size_t ws_bytes, void *stream);

/*
 * The paper's rule with work skipped that cannot change the result (section "Algorithm
 * Correctness": V_i is the AND over all j, so it is settled by the first j that eliminates i):
 * a victim that has met an eliminator is dropped from all further tests, while it goes on
 * eliminating others.  Same keep vector as nms_run_batched, bit for bit, from a fraction of the
 * pair tests on clustered detections (a quarter on 4096-box frames of SSD-style anchors).  One
 * workgroup per frame, which ranks the frame, keeps its boxes and the list of undecided victims in
 * LDS and takes the outranking boxes in stages of doubling width (with fewer frames than compute
 * units a frame's victims are shared out among several workgroups; frames beyond NMS_SORT_CHUNK
 * boxes always are, and their workgroups fetch the outranking boxes from the ranked table in
 * memory); it pays from about 2^28 pair slots per batch (frames * n_max^2) on.  Sizes as
 * nms_run_batched; workspace >= nms_workspace_bytes(n_max, frames), 256-byte aligned (used
 * for the rank step's tables unless the rank step runs inside the kernel; required in either case).
 * Arguments, layout, ownership and errors as nms_run_batched.
 */
int nms_run_early_exit_batched(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                               float threshold, uint8_t *keep_out, void *workspace, size_t ws_bytes, void *stream);

/*
 * The paper's own data layout, for measuring its form on this hardware: the boolean
 * matrix B as capacity x capacity BYTES over the UNSORTED input (Algorithm 1, one
 * matrix element per ordered pair, the score guard evaluated per pair), and
 * Algorithm 2's reduce with its k row partitions (a row gets capacity / k / 8 lanes --
 * capacity / k when that is not a multiple of 8 --, each of which folds its columns of all k
 * partitions; one combine per row instead of the paper's k block-wide ANDs).
 *   nms_map_matrix     B[i * capacity + j] = 0 iff j outranks i and overlap(i, j) >= theta,
 *                      else 1.  Every byte of B is written (the paper presets B to 1 with
 *                      a memset and rewrites the guarded entries; slots at or beyond n
 *                      never pass the guard there and come out as 1 here).
 *                      Outranking is this library's total order (index breaks score ties).
 *   nms_reduce_matrix  V[i] = AND over j of B[i * capacity + j], for all capacity rows
 *                      (rows of unused slots give 1, as in the paper).
 *   n <= capacity <= NMS_MAX_MATRIX, capacity a multiple of 64; k >= 1 divides capacity and
 *   capacity / k <= 1024; otherwise NMS_ERR_INVALID_ARG.
 */
int nms_map_matrix(const float *boxes, const float *scores, int n, int capacity, float threshold,
                   uint8_t *B, void *stream);
int nms_reduce_matrix(const uint8_t *B, int capacity, int k, uint8_t *V, void *stream);

/*
 * Profiling variant of the all-pairs routes (ranked or direct, chosen by size as in
 * nms_run_batched; never the early-exit route): identical work, and in addition records the
 * caller's HIP events on `stream`.  `events` is a HOST array of three hipEvent_t
 * (each may be NULL = skip): [0] before the rank step, [1] between rank and map,
 * [2] after the map step ([1] directly follows [0] on the direct route, which has no
 * rank step).  Event-record failures are reported as NMS_ERR_LAUNCH.
 */
int nms_run_batched_profiled(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                             float threshold, uint8_t *keep_out, void *workspace, size_t ws_bytes, void *stream,
                             void *const *events);

/*
 * nms_run: the same with the workspace taken from a pool registered once.
 * nms_init stores the pointer (caller-owned device memory, at least
 * nms_workspace_bytes(n_max, frames_max) bytes); nms_shutdown forgets it and never
 * frees it.  This pool is the library's only global state: one nms_run in flight at
 * a time, all on one stream.  nms_run before nms_init, or with n > the pool's n_max,
 * returns NMS_ERR_WORKSPACE.
 */
int nms_init(int n_max, int frames_max, void *workspace, size_t ws_bytes);
int nms_shutdown(void);
int nms_run(const float *boxes, const float *scores, int n, float threshold,
            uint8_t *keep_out, void *stream);

/*
 * nms_run_batched for callers that cannot allocate or bring scratch: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The workspace is a static
 * device array of NMS_STATIC_SCRATCH_BYTES inside the library (one copy per GPU, resident from
 * the time the library is loaded there until the process ends); the call makes no allocation
 * of any kind.  Same result as nms_run_batched, bit for bit; the caller still passes inputs
 * and keep_out.
 *   sizes    nms_workspace_bytes(n_max, frames) must not exceed NMS_STATIC_SCRATCH_BYTES, else
 *            NMS_ERR_TOO_LARGE and nothing is enqueued.  That admits any single frame the library
 *            takes (65,536 boxes: 3.3 MiB), 4 frames of 16,384 boxes, 23 of 4096, 92 of 1024.
 *   sharing  every call on a GPU uses that GPU's one array, which keeps the previous call's
 *            contents (nothing in it has to start at zero: each call writes what it reads).
 *            Calls on the same GPU must therefore be ordered on one stream; calls that overlap
 *            race.  Calls on different GPUs are independent (the current device selects the copy).
 *   set-up   the first call on a device looks up the array's address (hipGetSymbolAddress,
 *            once per device, under a lock); make that call outside graph capture.
 * Other arguments, layout, ownership and errors as nms_run_batched.
 */
int nms_run_static_batched(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                           float threshold, uint8_t *keep_out, void *stream);

/*
 * Host-only test hook: evaluates, on the CPU, the exact arithmetic the device pair
 * test uses for "does the outranking box eliminate the victim" (all pointers HOST:
 * victim[4], outranking[4]).  Every form of the test that a kernel may take for the pair is
 * evaluated (plain fast form; y-scaled; scaled late); returns 1/0, NMS_HOST_FORMS_DISAGREE if
 * they do not all give the same answer, or a negative status for a NaN threshold.
 * Lets the decision procedure be checked against plain division without a GPU.
 */
#define NMS_HOST_FORMS_DISAGREE (-100)
int nms_host_pair_test(const float *victim, const float *outranking, float threshold);

#ifdef __cplusplus
}
#endif
#endif /* NMS_MI355X_H */
