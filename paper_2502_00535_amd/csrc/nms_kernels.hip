// HIP kernels (gfx950, wave64) and the C ABI of the data-parallel NMS library.
//
// Steps (names follow the paper: D = detections, B = boolean matrix, V = survivors):
//   rank     total order on scores (Algorithm 1's guard "D[i].s < D[j].s", hoisted)
//   map      Algorithm 1 on the ranked lower triangle, one wavefront per 64x64 tile
//   reduce   Algorithm 2's row AND (here: row OR of elimination bits == 0)
//   fused    map with the row reduction folded in; no mask reaches memory
//
// Wave layout of the map step: lane = outranking box c of the tile's column block
// (its box and its per-box decision threshold live in VGPRs for the whole tile); the
// victim row r is wave-uniform and is fetched with scalar loads, so each victim costs
// 4 SGPRs and the 10 VALU instructions of the pair test.  The compare's lane mask IS the 64-bit
// elimination word of (row r, column block): no cross-lane work is needed to form it.
//
// This file is the one translation unit of the library: the kernels live in kernels/*.h
// (one file per step, included below inside the anonymous namespace), the launch logic and
// the extern "C" entry points follow.
#include <hip/hip_runtime.h>

#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>
#include <type_traits>

#include "../../include/nms.h"
#include "nms_pair.h"
#include "nms_host_logic.h"

// Scratch of nms_run_static_batched: one copy per GPU, held from the moment the library is
// loaded on it until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; the address the kernels use is static_scratch_on_current_device().
static __device__ __align__(256) unsigned char scratch[NMS_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kTile = NMS_TILE;
constexpr int kChunk = NMS_SORT_CHUNK;
constexpr unsigned long long kSentinel = ~0ull;

__device__ __forceinline__ int frame_count(const int32_t *counts, int f, int n_max)
{
    if (counts == nullptr) return n_max;
    int c = counts[f];
    return c < 0 ? 0 : (c > n_max ? n_max : c);
}

#include "kernels/rank.h"
#include "kernels/map.h"
#include "kernels/direct.h"
#include "kernels/reduce.h"
#include "kernels/greedy_sweep.h"
#include "kernels/greedy_walk.h"
#include "kernels/variants.h"
#include "kernels/early_exit.h"
#include "kernels/staged.h"
#include "kernels/small_frames.h"
#include "kernels/matrix_form.h"

// ----------------------------------------------------------------------------- host side

struct Pool {
    void *ws = nullptr;
    size_t bytes = 0;
    int n_max = 0;
    int frames_max = 0;
};
Pool g_pool;

inline size_t align256(size_t v) { return nms_align256(v); }

inline bool sizes_ok(int n_max, int frames, int *status)
{
    if (n_max < 0 || frames < 0) { *status = NMS_ERR_INVALID_ARG; return false; }
    if (n_max > NMS_MAX_N || frames > NMS_MAX_FRAMES) { *status = NMS_ERR_TOO_LARGE; return false; }
    // the map step is one launch of 256-thread workgroups, and a launch holds fewer than 2^32 threads
    const int T = nms_padded_n(n_max) / kTile;
    const bool super4 = (long long)frames * nms_triangle_units(T, 4) >= 16384;
    const long long tile_blocks = (nms_triangle_units(T, super4 ? 4 : 1) + kMapWaves - 1) / kMapWaves;
    const long long blocks = frames >= 8 ? (long long)((frames + 7) / 8) * 8 * tile_blocks : tile_blocks;
    if (blocks > NMS_MAX_MAP_WORKGROUPS) { *status = NMS_ERR_TOO_LARGE; return false; }
    return true;
}

inline bool is_nan(float v)
{
    uint32_t b;
    memcpy(&b, &v, sizeof b);
    return (b & 0x7fffffffu) > 0x7f800000u;
}

thread_local hipError_t g_last_hip_error = hipSuccess;

// The runtime's "last error" is per thread and sticky across libraries: an unrelated
// earlier failure (for example a probe made by the host framework) would otherwise be
// reported as ours.  begin_launch() discards it, launch_status() reads ours.
inline void begin_launch() { (void)hipGetLastError(); }

inline int launch_status()
{
    const hipError_t e = hipGetLastError();
    if (e == hipSuccess) return NMS_OK;
    g_last_hip_error = e;
    return NMS_ERR_LAUNCH;
}

int rank_launch(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                int32_t *order, float *sorted5, void *workspace, uint8_t *keep_preset, float4 *ysc, unsigned *ytile,
                hipStream_t stream, float *tsc = nullptr, double m = 0.0)
{
    const int n_pad = nms_padded_n(n_max);
    // one chunk up to kChunk boxes; beyond that, chunks of kMergeChunk (more workgroups, shorter sorts) and a merge
    const int n_chunks = n_max <= kChunk ? 1 : (n_max + kMergeChunk - 1) / kMergeChunk;
    int threads = 64;  // four keys per thread, at least one wavefront
    const int widest = n_max < kChunk ? n_max : kChunk;
    while (threads < 1024 && threads * 4 < widest) threads <<= 1;
    auto *keys_ws = static_cast<unsigned long long *>(workspace);
    begin_launch();
#define NMS_LAUNCH_RANK(P_, STAGE_)                                                                    \
    rank_chunk_kernel<P_, STAGE_><<<dim3(n_chunks, frames), dim3(P_ / 4), 0, stream>>>(                \
        boxes, scores, counts, n_max, n_pad, n_chunks, order, sorted5, keys_ws, keep_preset, ysc, ytile, tsc, m)
    if (n_chunks > 1) NMS_LAUNCH_RANK(kMergeChunk, false);
    else if (threads == 64) NMS_LAUNCH_RANK(256, true);
    else if (threads == 128) NMS_LAUNCH_RANK(512, true);
    else if (threads == 256) NMS_LAUNCH_RANK(1024, true);
    else if (threads == 512) NMS_LAUNCH_RANK(2048, true);
    else NMS_LAUNCH_RANK(4096, true);
#undef NMS_LAUNCH_RANK
    int st = launch_status();
    if (st != NMS_OK || n_chunks == 1) return st;
    begin_launch();
    rank_merge_kernel<<<dim3((n_pad * kMergeLanes + 255) / 256, frames), dim3(256), 0, stream>>>(
        boxes, counts, n_max, n_pad, n_chunks, keys_ws, order, sorted5, ysc, ytile, tsc, m);
    return launch_status();
}

int direct_launch(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                  float threshold, uint8_t *keep_out, hipStream_t stream)
{
    const NmsThetaConst th = nms_make_theta_const(threshold);
    const int tiles = (n_max + kTile - 1) / kTile;
    const int waves = tiles < 16 ? tiles : 16;
    // victims per workgroup: 16, or 8 / 4 when that is what it takes to have a workgroup for
    // every compute unit (a single 1024-box frame is 64 workgroups of 16 rows on a 256-CU chip)
    int rows = 16;
    while (rows > 4 && (long long)frames * ((n_max + rows - 1) / rows) < 256) rows >>= 1;
    const dim3 grid((n_max + rows - 1) / rows, frames);
    begin_launch();
#define NMS_LAUNCH_DIRECT(FAST_, ROWS_) \
    direct_kernel<FAST_, ROWS_><<<grid, dim3(waves * 64), 0, stream>>>(boxes, scores, counts, n_max, th, keep_out)
    if (th.fast) {
        if (rows == 16) NMS_LAUNCH_DIRECT(true, 16); else if (rows == 8) NMS_LAUNCH_DIRECT(true, 8); else NMS_LAUNCH_DIRECT(true, 4);
    } else {
        if (rows == 16) NMS_LAUNCH_DIRECT(false, 16); else if (rows == 8) NMS_LAUNCH_DIRECT(false, 8); else NMS_LAUNCH_DIRECT(false, 4);
    }
#undef NMS_LAUNCH_DIRECT
    return launch_status();
}

template <bool WRITE_MASK>
int map_launch(const float *sorted5, const int32_t *counts, int n_max, int frames, float threshold,
               unsigned long long *mask, const int32_t *order, uint8_t *keep_out, const float4 *ysc,
               const unsigned *ytile, hipStream_t stream)
{
    const int n_pad = nms_padded_n(n_max);
    const int T = n_pad / kTile;
    // four (or two) tiles per wavefront when that still leaves every SIMD several wavefronts
    const bool super4 = (long long)frames * nms_triangle_units(T, 4) >= 16384;
    const bool super2 = !super4 && (long long)frames * nms_triangle_units(T, 2) >= 16384;
    const int tiles = nms_triangle_units(T, super4 ? 4 : (super2 ? 2 : 1));  // work units, one per wavefront
    const NmsThetaConst th = nms_make_theta_const(threshold);
    const int tile_blocks = (tiles + kMapWaves - 1) / kMapWaves;
    // batches: one frame per XCD at a time (see the kernel); a few large frames: spread each over all XCDs
    const int xcd_frames = frames >= 8 ? 1 : 0;
    const dim3 grid = xcd_frames ? dim3((unsigned)(((frames + 7) / 8) * 8 * tile_blocks)) : dim3(tile_blocks, frames);
    const dim3 block(kMapWaves * 64);
    begin_launch();
#define NMS_LAUNCH_MAP(FAST_, SUPER_)                                                                             \
    map_tile_kernel<FAST_, WRITE_MASK, SUPER_><<<grid, block, 0, stream>>>(sorted5, counts, n_max, n_pad, tiles,  \
                                                                           tile_blocks, frames, xcd_frames, th,   \
                                                                           mask, order, keep_out, ysc, ytile)
    if (th.fast) {
        if (super4) NMS_LAUNCH_MAP(true, 4); else if (super2) NMS_LAUNCH_MAP(true, 2); else NMS_LAUNCH_MAP(true, 1);
    } else {
        if (super4) NMS_LAUNCH_MAP(false, 4); else if (super2) NMS_LAUNCH_MAP(false, 2); else NMS_LAUNCH_MAP(false, 1);
    }
#undef NMS_LAUNCH_MAP
    return launch_status();
}

}  // namespace

// ----------------------------------------------------------------------------- C ABI

extern "C" {

const char *nms_status_string(int status)
{
    switch (status) {
    case NMS_OK: return "ok";
    case NMS_ERR_INVALID_ARG: return "invalid argument";
    case NMS_ERR_TOO_LARGE: return "size beyond NMS_MAX_N or NMS_MAX_FRAMES";
    case NMS_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case NMS_ERR_LAUNCH: return "kernel launch failed";
    default: return "unknown status";
    }
}

int nms_version(void) { return NMS_VERSION; }

const char *nms_last_launch_error(void) { return hipGetErrorString(g_last_hip_error); }

int nms_padded_n(int n)
{
    if (n < 0 || n > NMS_MAX_N) return 0;
    return (n + kTile - 1) / kTile * kTile;
}

size_t nms_mask_words(int n)
{
    if (n < 0 || n > NMS_MAX_N) return 0;
    const size_t n_pad = (size_t)nms_padded_n(n);
    return (n_pad / kTile) * n_pad;
}

size_t nms_sort_workspace_bytes(int n_max, int frames)
{
    int st;
    if (!sizes_ok(n_max, frames, &st)) return 0;
    if (n_max <= kChunk) return 0;
    return align256((size_t)frames * nms_padded_n(n_max) * sizeof(unsigned long long));
}

size_t nms_workspace_bytes(int n_max, int frames)
{
    int st;
    if (!sizes_ok(n_max, frames, &st)) return 0;
    return nms_run_layout(n_max, nms_padded_n(n_max), frames, kChunk).end;
}

static_assert(kNmsRouteDirect == NMS_ROUTE_DIRECT && kNmsRouteAllPairs == NMS_ROUTE_ALL_PAIRS &&
                  kNmsRouteTwoLaunch == NMS_ROUTE_TWO_LAUNCH && kNmsRouteEarlyExit == NMS_ROUTE_EARLY_EXIT &&
                  kNmsRouteSmallFrames == NMS_ROUTE_SMALL_FRAMES,
              "route numbers of the header and of the host logic");

int nms_route(int n_max, int frames)
{
    int st;
    if (!sizes_ok(n_max, frames, &st) || n_max == 0 || frames == 0) return -1;
    return nms_route_for(n_max, frames, kChunk);
}

int nms_sort_batched(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                     int32_t *order, float *sorted5, void *workspace, size_t ws_bytes, void *stream)
{
    int st;
    if (!sizes_ok(n_max, frames, &st)) return st;
    if (n_max == 0 || frames == 0) return NMS_OK;
    if (!boxes || !scores || !order || !sorted5) return NMS_ERR_INVALID_ARG;
    const size_t need = nms_sort_workspace_bytes(n_max, frames);
    if (need != 0 && (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255))) return NMS_ERR_WORKSPACE;
    return rank_launch(boxes, scores, counts, n_max, frames, order, sorted5, workspace, nullptr, nullptr, nullptr,
                       static_cast<hipStream_t>(stream));
}

int nms_sort(const float *boxes, const float *scores, int n, int32_t *order, float *sorted5,
             void *workspace, size_t ws_bytes, void *stream)
{
    return nms_sort_batched(boxes, scores, nullptr, n, 1, order, sorted5, workspace, ws_bytes, stream);
}

int nms_overlap_mask_batched(const float *sorted5, const int32_t *counts, int n_max, int frames,
                             float threshold, uint64_t *mask, void *stream)
{
    int st;
    if (!sizes_ok(n_max, frames, &st)) return st;
    if (is_nan(threshold)) return NMS_ERR_INVALID_ARG;
    if (n_max == 0 || frames == 0) return NMS_OK;
    if (!sorted5 || !mask) return NMS_ERR_INVALID_ARG;
    return map_launch<true>(sorted5, counts, n_max, frames, threshold,
                            reinterpret_cast<unsigned long long *>(mask), nullptr, nullptr, nullptr, nullptr,
                            static_cast<hipStream_t>(stream));
}

int nms_overlap_mask(const float *sorted5, int n, float threshold, uint64_t *mask, void *stream)
{
    return nms_overlap_mask_batched(sorted5, nullptr, n, 1, threshold, mask, stream);
}

int nms_reduce_batched(const uint64_t *mask, const int32_t *order, const int32_t *counts, int n_max, int frames,
                       uint8_t *keep_out, void *stream)
{
    int st;
    if (!sizes_ok(n_max, frames, &st)) return st;
    if (n_max == 0 || frames == 0) return NMS_OK;
    if (!mask || !order || !keep_out) return NMS_ERR_INVALID_ARG;
    const int n_pad = nms_padded_n(n_max);
    begin_launch();
    const int row_pairs = (n_pad / kTile + 1) / 2;  // one wavefront per pair of tile rows, four per workgroup
    reduce_rows_kernel<<<dim3((row_pairs + 3) / 4, frames), dim3(256), 0, static_cast<hipStream_t>(stream)>>>(
        reinterpret_cast<const unsigned long long *>(mask), order, counts, n_max, n_pad, keep_out);
    return launch_status();
}

int nms_reduce(const uint64_t *mask, const int32_t *order, int n, uint8_t *keep_out, void *stream)
{
    return nms_reduce_batched(mask, order, nullptr, n, 1, keep_out, stream);
}

// Carve-up of the fused path's workspace (every part 256-byte aligned).
struct RunWorkspace {
    int32_t *order;     // [frames][n_max]
    float *sorted5;     // [frames][5 * n_pad]
    float4 *ysc;        // [frames][n_pad]       boxes with y * NMS_YSCALE, rank order
    unsigned *ytile;    // [frames][n_pad / 64]  1 = every box of the tile may use the y-scaled form
    float *tsc;         // [frames][n_pad]       NMS_YSCALE * T per box (fused map kernel)
    void *keys;         // rank scratch (n_max > NMS_SORT_CHUNK only)
    unsigned long long *stage;  // [frames][n_pad / 64][32] lane masks of the victims that each unit of the two-launch route's first launch eliminates (n_max > NMS_SORT_CHUNK only)
    char *end;
};

inline RunWorkspace carve_workspace(void *workspace, int n_max, int frames)
{
    const NmsRunLayout l = nms_run_layout(n_max, nms_padded_n(n_max), frames, kChunk);
    char *base = static_cast<char *>(workspace);
    RunWorkspace w;
    w.order = reinterpret_cast<int32_t *>(base + l.order);
    w.sorted5 = reinterpret_cast<float *>(base + l.sorted5);
    w.ysc = reinterpret_cast<float4 *>(base + l.ysc);
    w.ytile = reinterpret_cast<unsigned *>(base + l.ytile);
    w.tsc = reinterpret_cast<float *>(base + l.tsc);
    w.keys = base + l.keys;
    w.stage = reinterpret_cast<unsigned long long *>(base + l.stage);
    w.end = base + l.end;
    return w;
}

// The fused map step (map_fused_kernel): work units and grid as in map_launch.
static int fused_launch(const RunWorkspace &w, const int32_t *counts, int n_max, int frames, const NmsThetaConst &th,
                        uint8_t *keep_out, hipStream_t stream)
{
    const int n_pad = nms_padded_n(n_max);
    const int T = n_pad / kTile;
    const bool super4 = (long long)frames * nms_triangle_units(T, 4) >= 16384;
    const bool super2 = !super4 && (long long)frames * nms_triangle_units(T, 2) >= 16384;
    const int tiles = nms_triangle_units(T, super4 ? 4 : (super2 ? 2 : 1));
    const int tile_blocks = (tiles + kMapWaves - 1) / kMapWaves;
    const int xcd_frames = frames >= 8 ? 1 : 0;
    const dim3 grid = xcd_frames ? dim3((unsigned)(((frames + 7) / 8) * 8 * tile_blocks)) : dim3(tile_blocks, frames);
    const dim3 block(kMapWaves * 64);
    begin_launch();
#define NMS_LAUNCH_FUSED(FAST_, SUPER_)                                                                        \
    map_fused_kernel<FAST_, SUPER_><<<grid, block, 0, stream>>>(w.sorted5, counts, n_max, n_pad, tiles,        \
                                                                tile_blocks, frames, xcd_frames, th, w.order,  \
                                                                keep_out, w.ysc, w.ytile, w.tsc)
    if (th.fast) {
        if (super4) NMS_LAUNCH_FUSED(true, 4); else if (super2) NMS_LAUNCH_FUSED(true, 2); else NMS_LAUNCH_FUSED(true, 1);
    } else {
        if (super4) NMS_LAUNCH_FUSED(false, 4); else if (super2) NMS_LAUNCH_FUSED(false, 2); else NMS_LAUNCH_FUSED(false, 1);
    }
#undef NMS_LAUNCH_FUSED
    return launch_status();
}

// Frames of at most 1024 boxes: two stages of pair tests in one launch, no sort (kernels/small_frames.h).
static int small_frames_launch(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                               const NmsThetaConst &th, uint8_t *keep_out, hipStream_t stream)
{
    const int parts = nms_small_frames_parts(frames, n_max);
    const dim3 grid((unsigned)(frames * parts)), block(kSmallThreads);
    begin_launch();
    if (n_max <= kTinyThreads) {
        const dim3 tiny_block(kTinyThreads);
        if (th.fast)
            tiny_frames_kernel<true><<<grid, tiny_block, 0, stream>>>(boxes, scores, counts, n_max, parts, th, keep_out);
        else
            tiny_frames_kernel<false><<<grid, tiny_block, 0, stream>>>(boxes, scores, counts, n_max, parts, th, keep_out);
    } else if (n_max <= kSmallThreads) {
        if (th.fast)
            small_frames_kernel<true><<<grid, block, 0, stream>>>(boxes, scores, counts, n_max, parts, th, keep_out);
        else
            small_frames_kernel<false><<<grid, block, 0, stream>>>(boxes, scores, counts, n_max, parts, th, keep_out);
    } else if (n_max <= 2 * kSmallThreads) {
        if (th.fast)
            mid_frames_kernel<true, 2><<<grid, block, 0, stream>>>(boxes, scores, counts, n_max, parts, th, keep_out);
        else
            mid_frames_kernel<false, 2><<<grid, block, 0, stream>>>(boxes, scores, counts, n_max, parts, th, keep_out);
    } else {
        if (th.fast)
            mid_frames_kernel<true, 4><<<grid, block, 0, stream>>>(boxes, scores, counts, n_max, parts, th, keep_out);
        else
            mid_frames_kernel<false, 4><<<grid, block, 0, stream>>>(boxes, scores, counts, n_max, parts, th, keep_out);
    }
    return launch_status();
}

static int staged_launch(const RunWorkspace &w, const int32_t *counts, int n_max, int frames, const NmsThetaConst &th,
                         uint8_t *keep_out, hipStream_t stream)
{
    const int n_pad = nms_padded_n(n_max);
    const int T = n_pad / kTile;
    const dim3 first_grid((unsigned)(T * kStageTiles / kMapWaves), frames);
    int parts = 256 / frames;  // persistent workgroups of the second launch: one per compute unit (192 to 384 measure alike, 512: +3 %, 128: +18 %)
    if (parts < 1) parts = 1;
    begin_launch();
    if (th.fast)
        staged_first_kernel<true><<<first_grid, dim3(kMapWaves * 64), 0, stream>>>(w.sorted5, counts, n_max, n_pad, th, w.order,
                                                                                   keep_out, w.ysc, w.ytile, w.tsc, w.stage);
    else
        staged_first_kernel<false><<<first_grid, dim3(kMapWaves * 64), 0, stream>>>(w.sorted5, counts, n_max, n_pad, th, w.order,
                                                                                    keep_out, w.ysc, w.ytile, w.tsc, w.stage);
    int st = launch_status();
    if (st != NMS_OK) return st;
    begin_launch();
    if (th.fast)
        staged_second_kernel<true><<<dim3(parts, frames), dim3(kStageWaves * 64), 0, stream>>>(
            w.sorted5, counts, n_max, n_pad, th, w.order, keep_out, w.ysc, w.ytile, w.tsc, w.stage);
    else
        staged_second_kernel<false><<<dim3(parts, frames), dim3(kStageWaves * 64), 0, stream>>>(
            w.sorted5, counts, n_max, n_pad, th, w.order, keep_out, w.ysc, w.ytile, w.tsc, w.stage);
    return launch_status();
}

// forward: defined with the early-exit entry point below
static int early_exit_launch(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                             float threshold, uint8_t *keep_out, void *workspace, hipStream_t s);

// kRouteAuto: one launch for small frames, direct, all pairs, two launches or early exit by size (nms_route_for).  kRouteAllPairs: direct or ranked by size
// (every pair of the ranked triangle is evaluated).
enum Route { kRouteAuto = 0, kRouteRanked = 1, kRouteDirect = 2, kRouteAllPairs = 3 };

static int run_routed(Route route, const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                      float threshold, uint8_t *keep_out, void *workspace, size_t ws_bytes, void *stream,
                      void *const *events)
{
    int st;
    if (!sizes_ok(n_max, frames, &st)) return st;
    if (is_nan(threshold)) return NMS_ERR_INVALID_ARG;
    if (n_max == 0 || frames == 0) return NMS_OK;
    if (!boxes || !scores || !keep_out) return NMS_ERR_INVALID_ARG;
    const bool by_size = route == kRouteAuto || route == kRouteAllPairs;
    const bool small = route == kRouteAuto && nms_use_small_frames(n_max, frames);
    const bool direct = route == kRouteDirect || (by_size && !small && nms_use_direct_form(n_max, frames));
    if (route != kRouteDirect) {  // the automatic route validates the workspace whichever way it goes
        const size_t need = nms_workspace_bytes(n_max, frames);
        if (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255)) return NMS_ERR_WORKSPACE;
    }

    hipStream_t s = static_cast<hipStream_t>(stream);
    if (small)
        return small_frames_launch(boxes, scores, counts, n_max, frames, nms_make_theta_const(threshold), keep_out, s);
    if (route == kRouteAuto && !direct && nms_use_early_exit(n_max, frames, kChunk))
        return early_exit_launch(boxes, scores, counts, n_max, frames, threshold, keep_out, workspace, s);
    auto mark = [&](int i) {
        if (!events || !events[i]) return true;
        const hipError_t e = hipEventRecord(static_cast<hipEvent_t>(events[i]), s);
        if (e != hipSuccess) g_last_hip_error = e;
        return e == hipSuccess;
    };
    if (!mark(0)) return NMS_ERR_LAUNCH;
    if (direct) {
        if (!mark(1)) return NMS_ERR_LAUNCH;  // no rank step on this route
        st = direct_launch(boxes, scores, counts, n_max, frames, threshold, keep_out, s);
        if (st != NMS_OK) return st;
        return mark(2) ? NMS_OK : NMS_ERR_LAUNCH;
    }

    const RunWorkspace w = carve_workspace(workspace, n_max, frames);
    const NmsThetaConst th = nms_make_theta_const(threshold);
    const bool staged = route == kRouteAuto && nms_use_two_launches(n_max, frames, kChunk);
    st = rank_launch(boxes, scores, counts, n_max, frames, w.order, w.sorted5, w.keys, keep_out, w.ysc, w.ytile, s,
                     th.fast ? w.tsc : nullptr, th.m);
    if (st != NMS_OK) return st;
    if (!mark(1)) return NMS_ERR_LAUNCH;
    if (staged)
        st = staged_launch(w, counts, n_max, frames, th, keep_out, s);
    else
        st = fused_launch(w, counts, n_max, frames, th, keep_out, s);
    if (st != NMS_OK) return st;
    return mark(2) ? NMS_OK : NMS_ERR_LAUNCH;
}

int nms_run_batched_profiled(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                             float threshold, uint8_t *keep_out, void *workspace, size_t ws_bytes, void *stream,
                             void *const *events)
{
    return run_routed(kRouteAllPairs, boxes, scores, counts, n_max, frames, threshold, keep_out, workspace, ws_bytes,
                      stream, events);
}

int nms_run_batched(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                    float threshold, uint8_t *keep_out, void *workspace, size_t ws_bytes, void *stream)
{
    return run_routed(kRouteAuto, boxes, scores, counts, n_max, frames, threshold, keep_out, workspace, ws_bytes,
                      stream, nullptr);
}

int nms_run_ranked_batched(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                           float threshold, uint8_t *keep_out, void *workspace, size_t ws_bytes, void *stream)
{
    return run_routed(kRouteRanked, boxes, scores, counts, n_max, frames, threshold, keep_out, workspace, ws_bytes,
                      stream, nullptr);
}

int nms_run_direct_batched(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                           float threshold, uint8_t *keep_out, void *stream)
{
    return run_routed(kRouteDirect, boxes, scores, counts, n_max, frames, threshold, keep_out, nullptr, 0, stream,
                      nullptr);
}

int nms_reduce_greedy_batched(const uint64_t *mask, const int32_t *order, const int32_t *counts, int n_max,
                              int frames, uint8_t *keep_out, void *stream)
{
    int st;
    if (!sizes_ok(n_max, frames, &st)) return st;
    if (n_max == 0 || frames == 0) return NMS_OK;
    if (!mask || !order || !keep_out) return NMS_ERR_INVALID_ARG;
    const int n_pad = nms_padded_n(n_max);
    const int T = n_pad / kTile;
    const unsigned long long *m = reinterpret_cast<const unsigned long long *>(mask);
    hipStream_t s = static_cast<hipStream_t>(stream);
    for (int t0 = 0; t0 < T; t0 += kSweepTiles) {
        begin_launch();
        if (t0 == 0)
            greedy_sweep_kernel<true><<<dim3(frames), dim3(256), 0, s>>>(m, order, counts, n_max, n_pad, t0, keep_out);
        else
            greedy_sweep_kernel<false><<<dim3(frames), dim3(256), 0, s>>>(m, order, counts, n_max, n_pad, t0, keep_out);
        st = launch_status();
        if (st != NMS_OK) return st;
        const int later = T - (t0 + kSweepTiles);  // tile rows after this block
        if (later <= 0) break;
        const dim3 grid((later + 3) / 4, frames);
        begin_launch();
        if (t0 == 0)
            greedy_apply_kernel<true><<<grid, dim3(256), 0, s>>>(m, order, counts, n_max, n_pad, t0, keep_out);
        else
            greedy_apply_kernel<false><<<grid, dim3(256), 0, s>>>(m, order, counts, n_max, n_pad, t0, keep_out);
        st = launch_status();
        if (st != NMS_OK) return st;
    }
    return NMS_OK;
}

int nms_reduce_greedy(const uint64_t *mask, const int32_t *order, int n, uint8_t *keep_out, void *stream)
{
    return nms_reduce_greedy_batched(mask, order, nullptr, n, 1, keep_out, stream);
}

size_t nms_greedy_workspace_bytes(int n_max, int frames)
{
    int st;
    if (!sizes_ok(n_max, frames, &st)) return 0;
    return nms_workspace_bytes(n_max, frames) + align256((size_t)frames * nms_mask_words(n_max) * sizeof(uint64_t));
}

// rank, then greedy_fused_kernel (frames of at most NMS_SORT_CHUNK boxes)
static int run_greedy_fused(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                            float threshold, uint8_t *keep_out, void *workspace, hipStream_t s)
{
    const RunWorkspace w = carve_workspace(workspace, n_max, frames);
    int st = rank_launch(boxes, scores, counts, n_max, frames, w.order, w.sorted5, w.keys, nullptr, nullptr, nullptr, s);
    if (st != NMS_OK) return st;
    const NmsThetaConst th = nms_make_theta_const(threshold);
    const int n_pad = nms_padded_n(n_max);
    begin_launch();
    const FusedVariant none = {nullptr, nullptr, 0.0, 1.0f, 0};
    if (th.fast)
        greedy_fused_kernel<false, false, kExBoundary, false><<<dim3(frames), dim3(kFusedWaves * 64), 0, s>>>(
            w.sorted5, w.order, counts, n_max, n_pad, th, none, keep_out);
    else
        greedy_fused_kernel<false, false, kExDivideGe, false><<<dim3(frames), dim3(kFusedWaves * 64), 0, s>>>(
            w.sorted5, w.order, counts, n_max, n_pad, th, none, keep_out);
    return launch_status();
}

// The paper's rule with decided victims skipped (kernels/early_exit.h); arguments already validated.
static int early_exit_launch(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                             float threshold, uint8_t *keep_out, void *workspace, hipStream_t s)
{
    int st;
    const NmsThetaConst th = nms_make_theta_const(threshold);
    // Fewer frames than compute units: a frame's victims are shared out among `parts` workgroups
    // (each stages the whole frame), which then need the ranked table in memory.
    int parts = 1;
    while (parts < (n_max > kChunk ? 256 : 16) && frames * parts * 2 <= 256) parts *= 2;
    if (parts == 1 && n_max > kChunk / 2) {
        // the rank step would run with the same 1024 threads per frame: it is part of the kernel
        begin_launch();
        if (th.fast)
            early_exit_ranked_kernel<kPairFastYScaled><<<dim3(frames), dim3(kEarlyThreads), 0, s>>>(boxes, scores, counts, n_max, th,
                                                                                                    keep_out);
        else
            early_exit_ranked_kernel<kPairExact><<<dim3(frames), dim3(kEarlyThreads), 0, s>>>(boxes, scores, counts, n_max, th,
                                                                                              keep_out);
        return launch_status();
    }
    const RunWorkspace w = carve_workspace(workspace, n_max, frames);
    st = rank_launch(boxes, scores, counts, n_max, frames, w.order, w.sorted5, w.keys, nullptr, nullptr, nullptr, s);
    if (st != NMS_OK) return st;
    const int n_pad = nms_padded_n(n_max);
    if (n_max > kChunk) {
        // the frame's table does not fit LDS: every workgroup stages its share of the victims only
        while (parts * kChunk < n_max) parts *= 2;
        begin_launch();
        if (th.fast)
            early_exit_wide_kernel<kPairFast><<<dim3(frames * parts), dim3(kEarlyThreads), 0, s>>>(w.sorted5, w.order, counts, n_max,
                                                                                                   n_pad, parts, th, keep_out);
        else
            early_exit_wide_kernel<kPairExact><<<dim3(frames * parts), dim3(kEarlyThreads), 0, s>>>(w.sorted5, w.order, counts, n_max,
                                                                                                    n_pad, parts, th, keep_out);
        return launch_status();
    }
    begin_launch();
    if (th.fast)
        early_exit_kernel<kPairFastYScaled><<<dim3(frames * parts), dim3(kEarlyThreads), 0, s>>>(w.sorted5, w.order, counts, n_max,
                                                                                                 n_pad, parts, th, keep_out);
    else
        early_exit_kernel<kPairExact><<<dim3(frames * parts), dim3(kEarlyThreads), 0, s>>>(w.sorted5, w.order, counts, n_max, n_pad,
                                                                                           parts, th, keep_out);
    return launch_status();
}


int nms_run_early_exit_batched(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                               float threshold, uint8_t *keep_out, void *workspace, size_t ws_bytes, void *stream)
{
    int st;
    if (!sizes_ok(n_max, frames, &st)) return st;
    if (is_nan(threshold)) return NMS_ERR_INVALID_ARG;
    if (n_max == 0 || frames == 0) return NMS_OK;
    if (!boxes || !scores || !keep_out) return NMS_ERR_INVALID_ARG;
    if (!workspace || ws_bytes < nms_workspace_bytes(n_max, frames) || ((uintptr_t)workspace & 255))
        return NMS_ERR_WORKSPACE;
    return early_exit_launch(boxes, scores, counts, n_max, frames, threshold, keep_out, workspace,
                             static_cast<hipStream_t>(stream));
}

int nms_run_greedy_fused_batched(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                                 float threshold, uint8_t *keep_out, void *workspace, size_t ws_bytes, void *stream)
{
    int st;
    if (!sizes_ok(n_max, frames, &st)) return st;
    if (n_max > kChunk) return NMS_ERR_TOO_LARGE;
    if (is_nan(threshold)) return NMS_ERR_INVALID_ARG;
    if (n_max == 0 || frames == 0) return NMS_OK;
    if (!boxes || !scores || !keep_out) return NMS_ERR_INVALID_ARG;
    if (!workspace || ws_bytes < nms_workspace_bytes(n_max, frames) || ((uintptr_t)workspace & 255))
        return NMS_ERR_WORKSPACE;
    return run_greedy_fused(boxes, scores, counts, n_max, frames, threshold, keep_out, workspace,
                            static_cast<hipStream_t>(stream));
}

int nms_run_greedy_batched(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                           float threshold, uint8_t *keep_out, void *workspace, size_t ws_bytes, void *stream)
{
    int st;
    if (!sizes_ok(n_max, frames, &st)) return st;
    if (is_nan(threshold)) return NMS_ERR_INVALID_ARG;
    if (n_max == 0 || frames == 0) return NMS_OK;
    if (!boxes || !scores || !keep_out) return NMS_ERR_INVALID_ARG;
    if (!workspace || ws_bytes < nms_greedy_workspace_bytes(n_max, frames) || ((uintptr_t)workspace & 255))
        return NMS_ERR_WORKSPACE;
    // batches with a few dozen frames or more: one workgroup walks each frame, no mask
    // (measured crossover against rank + mask + sweep: 32 frames of 4096 boxes, 64 of 2048)
    if (n_max <= kChunk && (long long)frames * n_max >= kGreedyFusedBoxes)
        return run_greedy_fused(boxes, scores, counts, n_max, frames, threshold, keep_out, workspace,
                                static_cast<hipStream_t>(stream));
    const RunWorkspace w = carve_workspace(workspace, n_max, frames);
    unsigned long long *mask = reinterpret_cast<unsigned long long *>(w.end);
    int32_t *order = w.order;

    hipStream_t s = static_cast<hipStream_t>(stream);
    st = rank_launch(boxes, scores, counts, n_max, frames, w.order, w.sorted5, w.keys, nullptr, w.ysc, w.ytile, s);
    if (st != NMS_OK) return st;
    st = map_launch<true>(w.sorted5, counts, n_max, frames, threshold, mask, nullptr, nullptr, w.ysc, w.ytile, s);
    if (st != NMS_OK) return st;
    return nms_reduce_greedy_batched(reinterpret_cast<const uint64_t *>(mask), order, counts, n_max, frames, keep_out,
                                     stream);
}

size_t nms_ex_workspace_bytes(int n_max, int frames)
{
    int st;
    if (!sizes_ok(n_max, frames, &st)) return 0;
    return nms_greedy_workspace_bytes(n_max, frames)
         + 3 * align256((size_t)frames * nms_padded_n(n_max) * sizeof(float));  // ranked scores, labels, areas
}

int nms_run_ex_batched(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                       float threshold, const nms_options *options, uint8_t *keep_out,
                       void *workspace, size_t ws_bytes, void *stream)
{
    int st;
    if (!sizes_ok(n_max, frames, &st)) return st;
    if (is_nan(threshold)) return NMS_ERR_INVALID_ARG;
    nms_options opt = {NMS_RULE_PAPER, NMS_MEASURE_OUTRANKING_AREA, NMS_COMPARE_GE, NMS_TIES_BY_INDEX, 1.0f, 0, nullptr};
    if (options) opt = *options;
    if ((opt.rule | opt.measure | opt.compare | opt.ties) & ~1) return NMS_ERR_INVALID_ARG;
    if (opt.reserved != 0 || !(opt.pixel_offset == 0.0f || opt.pixel_offset == 1.0f)) return NMS_ERR_INVALID_ARG;
    if (n_max == 0 || frames == 0) return NMS_OK;
    if (!boxes || !scores || !keep_out) return NMS_ERR_INVALID_ARG;
    if (!workspace || ws_bytes < nms_ex_workspace_bytes(n_max, frames) || ((uintptr_t)workspace & 255))
        return NMS_ERR_WORKSPACE;
    // every option at its default: the default paths compute the same thing with fewer instructions
    if (opt.measure == NMS_MEASURE_OUTRANKING_AREA && opt.compare == NMS_COMPARE_GE && opt.ties == NMS_TIES_BY_INDEX &&
        opt.pixel_offset == 1.0f && opt.classes == nullptr) {
        if (opt.rule == NMS_RULE_PAPER)
            return nms_run_batched(boxes, scores, counts, n_max, frames, threshold, keep_out, workspace, ws_bytes, stream);
        return nms_run_greedy_batched(boxes, scores, counts, n_max, frames, threshold, keep_out, workspace, ws_bytes, stream);
    }

    const int n_pad = nms_padded_n(n_max);
    const RunWorkspace w = carve_workspace(workspace, n_max, frames);
    char *p = w.end;
    unsigned long long *mask = reinterpret_cast<unsigned long long *>(p);
    p += align256((size_t)frames * nms_mask_words(n_max) * sizeof(uint64_t));
    float *ranked_score = reinterpret_cast<float *>(p);
    p += align256((size_t)frames * n_pad * sizeof(float));
    int32_t *ranked_class = reinterpret_cast<int32_t *>(p);
    p += align256((size_t)frames * n_pad * sizeof(int32_t));
    float *ranked_area = reinterpret_cast<float *>(p);

    hipStream_t s = static_cast<hipStream_t>(stream);
    // under the paper's rule the row reduction is folded into the map kernel: keep_out starts at 1
    const bool fold = opt.rule == NMS_RULE_PAPER;
    st = rank_launch(boxes, scores, counts, n_max, frames, w.order, w.sorted5, w.keys, fold ? keep_out : nullptr, nullptr,
                     nullptr, s);
    if (st != NMS_OK) return st;
    begin_launch();
    gather_ranked_kernel<<<dim3((n_pad + 255) / 256, frames), dim3(256), 0, s>>>(
        w.order, scores, opt.classes, counts, w.sorted5, opt.pixel_offset, n_max, n_pad, ranked_score, ranked_class,
        ranked_area);
    st = launch_status();
    if (st != NMS_OK) return st;

    // work units and grid as in map_launch
    const int T = n_pad / kTile;
    const bool super4 = (long long)frames * nms_triangle_units(T, 4) >= 16384;
    const int tiles = nms_triangle_units(T, super4 ? 4 : 1);
    const int tile_blocks = (tiles + kMapWaves - 1) / kMapWaves;
    const int xcd_frames = frames >= 8 ? 1 : 0;
    const dim3 grid = xcd_frames ? dim3((unsigned)(((frames + 7) / 8) * 8 * tile_blocks)) : dim3(tile_blocks, frames);
    // rounding boundary of the division next to theta, exact in float64: below theta for ">=", above it for ">"
    double boundary = 0.0;
    bool divide = true;
    if (threshold >= 0x1p-40f && threshold <= 0x1p20f) {
        uint32_t bits;
        memcpy(&bits, &threshold, sizeof bits);
        const uint32_t other_bits = opt.compare == NMS_COMPARE_GT ? bits + 1u : bits - 1u;
        float other;
        memcpy(&other, &other_bits, sizeof other);
        boundary = 0.5 * ((double)threshold + (double)other);
        divide = false;
    }
    // a float32 at or below boundary * (1 - 2^-22): the factor of the variants kernel's first, float32 test
    float boundary_lo = 0.0f;
    if (!divide) {
        const double want = boundary * (1.0 - 0x1p-22);
        boundary_lo = (float)want;
        if ((double)boundary_lo > want) boundary_lo = nextafterf(boundary_lo, 0.0f);
    }
    const int flags = (opt.ties == NMS_TIES_IGNORE ? kExTiesIgnore : 0) | (opt.classes ? kExClasses : 0);
    const int mode = !divide ? kExBoundary : (opt.compare == NMS_COMPARE_GT ? kExDivideGt : kExDivideGe);
    const bool iou = opt.measure == NMS_MEASURE_IOU;
    const bool aux = flags != 0;
    if (opt.rule == NMS_RULE_GREEDY && n_max <= kChunk && (long long)frames * n_max >= kGreedyFusedBoxes) {
        // large batches under the greedy rule: the mask-free walk, one workgroup per frame
        const NmsThetaConst th = nms_make_theta_const(threshold);
        const FusedVariant v = {ranked_score, ranked_class, boundary, opt.pixel_offset, flags};
        begin_launch();
#define NMS_LAUNCH_WALK(IOU_, MODE_, AUX_)                                                          \
    greedy_fused_kernel<true, IOU_, MODE_, AUX_><<<dim3(frames), dim3(kFusedWaves * 64), 0, s>>>(   \
        w.sorted5, w.order, counts, n_max, n_pad, th, v, keep_out)
#define NMS_LAUNCH_WALK_MODE(IOU_, AUX_)                                                  \
    do {                                                                                  \
        if (mode == kExBoundary) NMS_LAUNCH_WALK(IOU_, kExBoundary, AUX_);                \
        else if (mode == kExDivideGe) NMS_LAUNCH_WALK(IOU_, kExDivideGe, AUX_);           \
        else NMS_LAUNCH_WALK(IOU_, kExDivideGt, AUX_);                                    \
    } while (0)
        if (iou) {
            if (aux) NMS_LAUNCH_WALK_MODE(true, true); else NMS_LAUNCH_WALK_MODE(true, false);
        } else {
            if (aux) NMS_LAUNCH_WALK_MODE(false, true); else NMS_LAUNCH_WALK_MODE(false, false);
        }
#undef NMS_LAUNCH_WALK_MODE
#undef NMS_LAUNCH_WALK
        return launch_status();
    }
    begin_launch();
#define NMS_LAUNCH_EX_SUPER(IOU_, MODE_, AUX_, SUPER_, MASK_)                                                     \
    map_tile_ex_kernel<IOU_, MODE_, AUX_, SUPER_, MASK_><<<grid, dim3(kMapWaves * 64), 0, s>>>(                   \
        w.sorted5, ranked_score, ranked_class, ranked_area, counts, n_max, n_pad, tiles, tile_blocks, frames,     \
        xcd_frames, threshold, boundary, boundary_lo, opt.pixel_offset, flags, mask, w.order, keep_out)
#define NMS_LAUNCH_EX(IOU_, MODE_, AUX_)                                                  \
    do {                                                                                  \
        if (fold) {                                                                       \
            if (super4) NMS_LAUNCH_EX_SUPER(IOU_, MODE_, AUX_, 4, false);                 \
            else NMS_LAUNCH_EX_SUPER(IOU_, MODE_, AUX_, 1, false);                        \
        } else {                                                                          \
            if (super4) NMS_LAUNCH_EX_SUPER(IOU_, MODE_, AUX_, 4, true);                  \
            else NMS_LAUNCH_EX_SUPER(IOU_, MODE_, AUX_, 1, true);                         \
        }                                                                                 \
    } while (0)
#define NMS_LAUNCH_EX_MODE(IOU_, AUX_)                                                    \
    do {                                                                                  \
        if (mode == kExBoundary) NMS_LAUNCH_EX(IOU_, kExBoundary, AUX_);                  \
        else if (mode == kExDivideGe) NMS_LAUNCH_EX(IOU_, kExDivideGe, AUX_);             \
        else NMS_LAUNCH_EX(IOU_, kExDivideGt, AUX_);                                      \
    } while (0)
    if (iou) {
        if (aux) NMS_LAUNCH_EX_MODE(true, true); else NMS_LAUNCH_EX_MODE(true, false);
    } else {
        if (aux) NMS_LAUNCH_EX_MODE(false, true); else NMS_LAUNCH_EX_MODE(false, false);
    }
#undef NMS_LAUNCH_EX_MODE
#undef NMS_LAUNCH_EX_SUPER
#undef NMS_LAUNCH_EX
    st = launch_status();
    if (st != NMS_OK) return st;
    if (fold) return NMS_OK;
    return nms_reduce_greedy_batched(reinterpret_cast<const uint64_t *>(mask), w.order, counts, n_max, frames,
                                     keep_out, stream);
}

int nms_map_matrix(const float *boxes, const float *scores, int n, int capacity, float threshold,
                   uint8_t *B, void *stream)
{
    if (n < 0 || capacity < 0) return NMS_ERR_INVALID_ARG;
    if (capacity > NMS_MAX_MATRIX) return NMS_ERR_TOO_LARGE;
    if (n > capacity || capacity % kTile != 0 || is_nan(threshold)) return NMS_ERR_INVALID_ARG;
    if (capacity == 0) return NMS_OK;
    if (!B || (n > 0 && (!boxes || !scores))) return NMS_ERR_INVALID_ARG;
    const NmsThetaConst th = nms_make_theta_const(threshold);
    const dim3 grid((capacity + 255) / 256, (capacity + 4 * kMatRows - 1) / (4 * kMatRows));
    hipStream_t s = static_cast<hipStream_t>(stream);
    begin_launch();
    if (th.fast)
        map_matrix_kernel<true><<<grid, dim3(256), 0, s>>>(boxes, scores, n, capacity, th, B);
    else
        map_matrix_kernel<false><<<grid, dim3(256), 0, s>>>(boxes, scores, n, capacity, th, B);
    return launch_status();
}

int nms_reduce_matrix(const uint8_t *B, int capacity, int k, uint8_t *V, void *stream)
{
    if (capacity < 0 || k < 1) return NMS_ERR_INVALID_ARG;
    if (capacity > NMS_MAX_MATRIX) return NMS_ERR_TOO_LARGE;
    if (capacity % kTile != 0) return NMS_ERR_INVALID_ARG;
    if (capacity == 0) return NMS_OK;
    if (capacity % k != 0 || capacity / k > 1024 || !B || !V) return NMS_ERR_INVALID_ARG;
    const int part = capacity / k;
    const int vec = part % 8 == 0 ? 8 : 1;                       // bytes per load
    const int waves_per_row = (part / vec + 63) / 64;             // 1 .. 16
    const int block_waves = waves_per_row <= 4 ? 4 : waves_per_row;
    const int rows_per_block = block_waves / waves_per_row;
    const dim3 grid((capacity + rows_per_block - 1) / rows_per_block);
    hipStream_t s = static_cast<hipStream_t>(stream);
    begin_launch();
    if (vec == 8)
        reduce_matrix_kernel<8><<<grid, dim3(block_waves * 64), 0, s>>>(B, capacity, k, waves_per_row, V);
    else
        reduce_matrix_kernel<1><<<grid, dim3(block_waves * 64), 0, s>>>(B, capacity, k, waves_per_row, V);
    return launch_status();
}

int nms_run_ws(const float *boxes, const float *scores, int n, float threshold,
               uint8_t *keep_out, void *workspace, size_t ws_bytes, void *stream)
{
    return nms_run_batched(boxes, scores, nullptr, n, 1, threshold, keep_out, workspace, ws_bytes, stream);
}

int nms_init(int n_max, int frames_max, void *workspace, size_t ws_bytes)
{
    int st;
    if (!sizes_ok(n_max, frames_max, &st)) return st;
    if (n_max == 0 || frames_max == 0) return NMS_ERR_INVALID_ARG;
    if (!workspace || ((uintptr_t)workspace & 255) || ws_bytes < nms_workspace_bytes(n_max, frames_max))
        return NMS_ERR_WORKSPACE;
    g_pool.ws = workspace;
    g_pool.bytes = ws_bytes;
    g_pool.n_max = n_max;
    g_pool.frames_max = frames_max;
    return NMS_OK;
}

int nms_shutdown(void)
{
    g_pool = Pool();
    return NMS_OK;
}

int nms_run(const float *boxes, const float *scores, int n, float threshold, uint8_t *keep_out, void *stream)
{
    int st;
    if (!sizes_ok(n, 1, &st)) return st;
    if (is_nan(threshold)) return NMS_ERR_INVALID_ARG;
    if (n == 0) return NMS_OK;
    if (!g_pool.ws || n > g_pool.n_max) return NMS_ERR_WORKSPACE;
    return nms_run_batched(boxes, scores, nullptr, n, 1, threshold, keep_out, g_pool.ws, g_pool.bytes, stream);
}

// Device address of `scratch` on the current GPU, looked up once per device.
static int static_scratch_on_current_device(void **out)
{
    constexpr int kMaxDevices = 64;
    static std::mutex lock;
    static void *address[kMaxDevices] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { g_last_hip_error = e; return NMS_ERR_LAUNCH; }
    if (dev < 0 || dev >= kMaxDevices) return NMS_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> hold(lock);
    if (address[dev] == nullptr) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || p == nullptr) {
            g_last_hip_error = e != hipSuccess ? e : hipErrorInvalidSymbol;
            (void)hipGetLastError();
            return NMS_ERR_LAUNCH;
        }
        address[dev] = p;
    }
    *out = address[dev];
    return NMS_OK;
}

int nms_run_static_batched(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                           float threshold, uint8_t *keep_out, void *stream)
{
    int st;
    if (!sizes_ok(n_max, frames, &st)) return st;
    if (is_nan(threshold)) return NMS_ERR_INVALID_ARG;
    if (n_max == 0 || frames == 0) return NMS_OK;
    if (!boxes || !scores || !keep_out) return NMS_ERR_INVALID_ARG;
    if (nms_workspace_bytes(n_max, frames) > (size_t)NMS_STATIC_SCRATCH_BYTES) return NMS_ERR_TOO_LARGE;
    void *ws = nullptr;
    st = static_scratch_on_current_device(&ws);
    if (st != NMS_OK) return st;
    return run_routed(kRouteAuto, boxes, scores, counts, n_max, frames, threshold, keep_out, ws,
                      (size_t)NMS_STATIC_SCRATCH_BYTES, stream, nullptr);
}

int nms_host_pair_test(const float *victim, const float *outranking, float threshold)
{
    if (!victim || !outranking || is_nan(threshold)) return NMS_ERR_INVALID_ARG;
    const NmsThetaConst th = nms_make_theta_const(threshold);
    const float a = nms_box_area(outranking[0], outranking[1], outranking[2], outranking[3]);
    if (!th.fast)
        return nms_eliminates_exact(victim[0], victim[1], victim[2], victim[3], outranking[0], outranking[1], outranking[2],
                                    outranking[3], a, th.theta) ? 1 : 0;
    // every fast form that the kernels may take for this pair; they have to agree
    const float T = nms_pair_threshold(a, th.m);
    const bool hit = nms_eliminates_fast(victim[0], victim[1], victim[2], victim[3],
                                         outranking[0], outranking[1], outranking[2], outranking[3], T);
    const bool regular = nms_y_regular(victim[1]) && nms_y_regular(victim[3]) && nms_y_regular(outranking[1]) &&
                         nms_y_regular(outranking[3]);
    if (regular &&  // what the fused kernel does for a pair of regular tiles
        hit != nms_eliminates_fast_yscaled(victim[0], victim[1] * NMS_YSCALE, victim[2], victim[3] * NMS_YSCALE,
                                           outranking[0], outranking[1] * NMS_YSCALE, outranking[2],
                                           outranking[3] * NMS_YSCALE, T * NMS_YSCALE, NMS_YSCALE))
        return NMS_HOST_FORMS_DISAGREE;
    if (nms_extent_fits_late_scaling(outranking[1], outranking[3]) &&
        hit != nms_eliminates_fast_latescaled(victim[0], victim[1], victim[2], victim[3], outranking[0], outranking[1],
                                              outranking[2], outranking[3], T * NMS_YSCALE, NMS_YSCALE))
        return NMS_HOST_FORMS_DISAGREE;
    return hit ? 1 : 0;
}

}  // extern "C"
