// Part of nms_kernels.hip (included there, inside its anonymous namespace): rank step: radix sort of a chunk in LDS, merge of several chunks.
#pragma once

// ----------------------------------------------------------------------------- rank

// Sort keys: nms_rank_key in nms_host_logic.h (unique, ascending = better score first, then lower index).

// Rank-ordered row r: the box and its area, and (fused path only, ysc != nullptr) the same
// box with y multiplied by NMS_YSCALE.  Returns whether the box may use the y-scaled form.
// The fused map kernel also gets, per box, the float32 that intersections with it are compared
// with, already multiplied by NMS_YSCALE (tsc_f; m = the rounding boundary below the threshold,
// 0 when the threshold takes the literal division and the table is not used).
__device__ __forceinline__ bool emit_ranked_box(const float4 b, int idx, int r, int n_pad,
                                               int32_t *order_f, float *sorted_f, float4 *ysc_f, float *tsc_f, double m)
{
    order_f[r] = idx;
    reinterpret_cast<float4 *>(sorted_f)[r] = b;
    const float area = nms_box_area(b.x, b.y, b.z, b.w);
    sorted_f[4 * (size_t)n_pad + r] = area;
    if (ysc_f != nullptr) ysc_f[r] = make_float4(b.x, b.y * NMS_YSCALE, b.z, b.w * NMS_YSCALE);
    if (tsc_f != nullptr) tsc_f[r] = nms_pair_threshold(area, m) * NMS_YSCALE;
    return nms_y_regular(b.y) && nms_y_regular(b.w);
}

__device__ __forceinline__ void emit_padding_row(int r, int n_pad, float *sorted_f, float4 *ysc_f, float *tsc_f)
{
    reinterpret_cast<float4 *>(sorted_f)[r] = make_float4(0.f, 0.f, 0.f, 0.f);
    sorted_f[4 * (size_t)n_pad + r] = 1.0f;  // the one-pixel box (0,0,0,0): never divides by zero
    if (ysc_f != nullptr) ysc_f[r] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (tsc_f != nullptr) tsc_f[r] = INFINITY;  // no intersection reaches it
}

// Inclusive prefix sum over the 64 lanes of a wavefront with DPP: shifts by 1, 2, 4, 8 inside
// each row of 16 lanes (lanes shifted in from outside a row read 0), then lane 15 of each row
// broadcast into the next row (rows 1 and 3), then lane 31 into rows 2 and 3.
__device__ __forceinline__ unsigned wave_inclusive_sum(unsigned x)
{
    x += (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xf, 0xf, true);  // row_shr:1
    x += (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xf, 0xf, true);  // row_shr:2
    x += (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xf, 0xf, true);  // row_shr:4
    x += (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xf, 0xf, true);  // row_shr:8
    x += (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x142, 0xa, 0xf, false); // row_bcast:15 into rows 1, 3
    x += (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x143, 0xc, 0xf, false); // row_bcast:31 into rows 2, 3
    return x;
}

// The same inside each row of 16 lanes only (the first four steps).
__device__ __forceinline__ unsigned row16_inclusive_sum(unsigned x)
{
    x += (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xf, 0xf, true);  // row_shr:1
    x += (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xf, 0xf, true);  // row_shr:2
    x += (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xf, 0xf, true);  // row_shr:4
    x += (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xf, 0xf, true);  // row_shr:8
    return x;
}

// The minimum over each row of 16 lanes, in every lane of the row (rotations inside the row).
__device__ __forceinline__ unsigned row16_min(unsigned x)
{
    unsigned y;
    y = (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x121, 0xf, 0xf, false);  // row_ror:1
    x = y < x ? y : x;
    y = (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x122, 0xf, 0xf, false);  // row_ror:2
    x = y < x ? y : x;
    y = (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x124, 0xf, 0xf, false);  // row_ror:4
    x = y < x ? y : x;
    y = (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x128, 0xf, 0xf, false);  // row_ror:8
    x = y < x ? y : x;
    return x;
}

// Stable LSD radix sort of the P = 4 * blockDim.x (key, index) pairs of a workgroup, eight
// bits per pass, four passes.  Element e = 256 * wave + 64 * q + lane is register q of its
// thread.  Stability is what makes 32-bit keys enough: elements start in index order, so
// equal scores keep the lower index first (the tie rule) without the index taking part in
// any compare.  Per pass:
//   - every wavefront ranks its 256 elements among themselves.  The lanes that hold the same
//     digit find each other through tables of 256 lane masks: every lane ORs its bit into the
//     entry of its digit (an LDS atomic; OR does not care in which order) and reads the entry
//     back; the mask's first lane clears the entry again, so a table is all zero between uses.
//     An element stands behind the elements of earlier registers q with its digit and behind
//     the lower lanes of its own mask; the first lane of each mask adds the mask's population
//     to a per-wavefront histogram in LDS, touched by its own wavefront only.  (A wavefront's
//     LDS instructions execute in order, so no barrier is needed inside a wavefront.)
//   - the histograms are turned into start offsets per (digit, wavefront);
//   - every element goes to start + place in `buf`, and the threads read their elements back.
// After the last pass `buf` holds ((key << 32) | index) in sorted order.
//
// Workgroups of at most four wavefronts (W = blockDim.x / 64): two barriers per pass.
//   - a wavefront keeps one table of lane masks per register q, so the four ORs and the reads are
//     issued together: element (q, lane) with digit d stands behind the population counts of the
//     masks of earlier q at d;
//   - after the barrier every wavefront turns the W histograms into its own start offsets (lane l
//     takes digits 4l .. 4l+3: totals over the wavefronts, prefix sum across the lanes, plus the
//     counts of the wavefronts before its own) and keeps them in a row of its own, so the scatter
//     follows without another barrier.
// match: W x 4 x 256 lane masks; hist, wbase: W x 256 counters each.
template <int W>
__device__ __forceinline__ void radix_rank_small(unsigned (&key)[4], unsigned (&idx)[4], const int (&e)[4],
                                                 unsigned long long *buf, unsigned *hist, unsigned *wbase,
                                                 unsigned long long *match)
{
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    unsigned *myhist = hist + wave * 256;
    unsigned *mybase = wbase + wave * 256;
    unsigned long long *mytab = match + wave * 1024;
    for (int i = lane; i < 1024; i += 64) mytab[i] = 0ull;
#pragma unroll 1
    for (int shift = 0; shift < 32; shift += 8) {
        reinterpret_cast<uint4 *>(myhist)[lane] = make_uint4(0u, 0u, 0u, 0u);
        unsigned d[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            d[q] = (key[q] >> shift) & 255u;
            __hip_atomic_fetch_or(&mytab[q * 256 + d[q]], 1ull << lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
        }
        // a wavefront's LDS instructions execute in order: the fence only keeps the compiler from moving the reads up
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        unsigned long long own[4];
        unsigned before[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            before[q] = 0;
#pragma unroll
            for (int p = 0; p < q; ++p)
                before[q] += (unsigned)__popcll(__hip_atomic_load(&mytab[p * 256 + d[q]], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT));
            own[q] = __hip_atomic_load(&mytab[q * 256 + d[q]], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        unsigned place[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const unsigned m_lo = (unsigned)own[q], m_hi = (unsigned)(own[q] >> 32);
            const unsigned below = __builtin_amdgcn_mbcnt_hi(m_hi, __builtin_amdgcn_mbcnt_lo(m_lo, 0u));
            place[q] = before[q] + below;
            if (below == 0) {
                __hip_atomic_fetch_add(&myhist[d[q]], __popc(m_lo) + __popc(m_hi), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
                __hip_atomic_store(&mytab[q * 256 + d[q]], 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
            }
        }
        __syncthreads();
        {
            uint4 h[W];
#pragma unroll
            for (int w = 0; w < W; ++w) h[w] = reinterpret_cast<const uint4 *>(hist + w * 256)[lane];
            uint4 all = make_uint4(0u, 0u, 0u, 0u), pre = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
            for (int w = 0; w < W; ++w) {
                if (w < wave) { pre.x += h[w].x; pre.y += h[w].y; pre.z += h[w].z; pre.w += h[w].w; }
                all.x += h[w].x; all.y += h[w].y; all.z += h[w].z; all.w += h[w].w;
            }
            const unsigned sum = all.x + all.y + all.z + all.w;
            const unsigned excl = wave_inclusive_sum(sum) - sum;
            reinterpret_cast<uint4 *>(mybase)[lane] = make_uint4(excl + pre.x, excl + all.x + pre.y, excl + all.x + all.y + pre.z,
                                                                 excl + all.x + all.y + all.z + pre.w);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const unsigned dest = __hip_atomic_load(&mybase[d[q]], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT) + place[q];
            buf[dest] = ((unsigned long long)key[q] << 32) | idx[q];
        }
        __syncthreads();
        if (shift < 24) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const unsigned long long v = buf[e[q]];
                key[q] = (unsigned)(v >> 32);
                idx[q] = (unsigned)v;
            }
        }
    }
}

// The same sort for workgroups of eight or sixteen wavefronts (2048 or 4096 elements), where four
// lane-mask tables per wavefront do not fit LDS: two tables, the registers in two rounds (0 and 1,
// then 2 and 3).  The second round finds the elements of the first round with its digit in the
// wavefront's histogram (a wavefront's LDS operations execute in order, so the first round's counts
// are there).  The digit totals are summed over the wavefronts by the first 256 threads (a thread
// per digit, all its reads issued together); the prefix sum over the 256 totals is then done by every wavefront for itself
// (one 16-byte read per lane, a DPP scan) and added to its own histogram row, so that the scatter
// follows without a third barrier: three per pass instead of four.
// match: W x 2 x 256 lane masks; hist, wbase: W x 256 counters each; tot: 256.
template <int W>
__device__ __forceinline__ void radix_rank_large(unsigned (&key)[4], unsigned (&idx)[4], const int (&e)[4],
                                                 unsigned long long *buf, unsigned *hist, unsigned *tot, unsigned *wbase,
                                                 unsigned long long *match)
{
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    unsigned *myhist = hist + wave * 256;
    unsigned *mybase = wbase + wave * 256;
    unsigned long long *tab0 = match + wave * 512;
    unsigned long long *tab1 = tab0 + 256;
    for (int i = lane; i < 512; i += 64) tab0[i] = 0ull;
    auto or_bit = [&](unsigned long long *t, unsigned d) __attribute__((always_inline)) {
        __hip_atomic_fetch_or(&t[d], 1ull << lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
    };
    auto load_mask = [&](unsigned long long *t, unsigned d) __attribute__((always_inline)) {
        return __hip_atomic_load(&t[d], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
    };
    auto below_in = [&](unsigned long long m) __attribute__((always_inline)) {
        return __builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)m, 0u));
    };
    // the first lane of a mask adds its population to the histogram and clears the entry
    auto settle = [&](unsigned long long *t, unsigned d, unsigned long long m, unsigned below) __attribute__((always_inline)) {
        if (below == 0) {
            __hip_atomic_fetch_add(&myhist[d], (unsigned)__popcll(m), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
            __hip_atomic_store(&t[d], 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
        }
    };
#pragma unroll 1
    for (int shift = 0; shift < 32; shift += 8) {
        reinterpret_cast<uint4 *>(myhist)[lane] = make_uint4(0u, 0u, 0u, 0u);
        unsigned d[4], place[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) d[q] = (key[q] >> shift) & 255u;
        // (the fences only keep the compiler from reordering: a wavefront's LDS instructions execute in order)
        or_bit(tab0, d[0]);
        or_bit(tab1, d[1]);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        {
            const unsigned long long m0 = load_mask(tab0, d[0]);
            const unsigned long long m01 = load_mask(tab0, d[1]);
            const unsigned long long m1 = load_mask(tab1, d[1]);
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            const unsigned b0 = below_in(m0), b1 = below_in(m1);
            place[0] = b0;
            place[1] = (unsigned)__popcll(m01) + b1;
            settle(tab0, d[0], m0, b0);
            settle(tab1, d[1], m1, b1);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        or_bit(tab0, d[2]);
        or_bit(tab1, d[3]);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        {
            const unsigned h2 = __hip_atomic_load(&myhist[d[2]], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
            const unsigned h3 = __hip_atomic_load(&myhist[d[3]], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
            const unsigned long long m2 = load_mask(tab0, d[2]);
            const unsigned long long m23 = load_mask(tab0, d[3]);
            const unsigned long long m3 = load_mask(tab1, d[3]);
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            const unsigned b2 = below_in(m2), b3 = below_in(m3);
            place[2] = h2 + b2;
            place[3] = h3 + (unsigned)__popcll(m23) + b3;
            settle(tab0, d[2], m2, b2);
            settle(tab1, d[3], m3, b3);
        }
        __syncthreads();
        if (tid < 256) {
            // the counts of digit tid in every wavefront (all reads issued together), then their running sums
            unsigned t[W];
#pragma unroll
            for (int w = 0; w < W; ++w) t[w] = hist[w * 256 + tid];
            unsigned run = 0;
#pragma unroll
            for (int w = 0; w < W; ++w) {
                hist[w * 256 + tid] = run;
                run += t[w];
            }
            tot[tid] = run;
        }
        __syncthreads();
        {
            const uint4 all = reinterpret_cast<const uint4 *>(tot)[lane];
            const uint4 pre = reinterpret_cast<const uint4 *>(myhist)[lane];
            const unsigned sum = all.x + all.y + all.z + all.w;
            const unsigned excl = wave_inclusive_sum(sum) - sum;
            reinterpret_cast<uint4 *>(mybase)[lane] = make_uint4(excl + pre.x, excl + all.x + pre.y, excl + all.x + all.y + pre.z,
                                                                 excl + all.x + all.y + all.z + pre.w);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const unsigned dest = __hip_atomic_load(&mybase[d[q]], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT) + place[q];
            buf[dest] = ((unsigned long long)key[q] << 32) | idx[q];
        }
        __syncthreads();
        if (shift < 24) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const unsigned long long v = buf[e[q]];
                key[q] = (unsigned)(v >> 32);
                idx[q] = (unsigned)v;
            }
        }
    }
}

// One workgroup ranks one chunk of up to kChunk boxes of one frame: P = 4 * blockDim.x
// elements (P a multiple of 256, 256..4096), four per thread, sorted by radix_rank_small or radix_rank_large.
// With a single chunk the kernel also writes order / sorted5 (and, for the fused path,
// presets keep_out); with several chunks it leaves the chunk's sorted keys in `keys_ws`
// for the merge kernel.
// STAGE (single chunk): the boxes are fetched in input order, coalesced, together with the
// scores, wait in registers while the sort runs and change hands through LDS afterwards --
// instead of a second, dependent round trip to memory for a gather by rank.
template <int P, bool STAGE>
__global__ void __launch_bounds__(P / 4)
rank_chunk_kernel(const float *__restrict__ boxes, const float *__restrict__ scores,
                  const int32_t *__restrict__ counts, int n_max, int n_pad, int n_chunks,
                  int32_t *__restrict__ order, float *__restrict__ sorted5,
                  unsigned long long *__restrict__ keys_ws, uint8_t *__restrict__ keep_preset,
                  float4 *__restrict__ ysc, unsigned *__restrict__ ytile, float *__restrict__ tsc, double m)
{
    __shared__ unsigned long long keys[P];
    __shared__ __align__(16) unsigned hist[(P / 256) * 256];  // one row of 256 digit counts per wavefront
    __shared__ __align__(16) unsigned tot[256];
    constexpr bool kSmall = P <= 1024;  // at most four wavefronts: radix_rank_small
    __shared__ float4 stage[kSmall ? 2 * P : (STAGE ? P : P / 2)];  // during the sort: the wavefronts' lane-mask tables (P x 16 bytes; P x 32 for radix_rank_small)
    __shared__ __align__(16) unsigned wbase[P];  // one row of 256 start offsets per wavefront
    const int f = blockIdx.y;
    const int chunk = blockIdx.x;
    const int tid = threadIdx.x;
    const int nth = blockDim.x;
    const int lane = tid & 63;
    const int n_f = frame_count(counts, f, n_max);
    constexpr int kSpan = STAGE ? kChunk : P;  // boxes per chunk: several chunks are P boxes each
    const int base = chunk * kSpan;
    int cnt = n_f - base;
    cnt = cnt < 0 ? 0 : (cnt > kSpan ? kSpan : cnt);
    const float *scores_f = scores + (size_t)f * n_max;
    const float *boxes_f = boxes + (size_t)f * n_max * 4;
    int e[4];
    unsigned long long K[4];
    float4 mine[4];  // STAGE: box e[q] of the input
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        e[q] = (tid >> 6) * 256 + q * 64 + lane;
        K[q] = (e[q] < cnt) ? nms_rank_key(scores_f[base + e[q]], (unsigned)(base + e[q])) : kSentinel;
        if (STAGE) mine[q] = (e[q] < cnt) ? reinterpret_cast<const float4 *>(boxes_f)[e[q]] : make_float4(0.f, 0.f, 0.f, 0.f);
    }

    unsigned key32[4], index[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        key32[q] = (unsigned)(K[q] >> 32);
        index[q] = (unsigned)K[q];
    }
    if constexpr (kSmall)
        radix_rank_small<P / 256>(key32, index, e, keys, hist, wbase, reinterpret_cast<unsigned long long *>(stage));
    else
        radix_rank_large<P / 256>(key32, index, e, keys, hist, tot, wbase, reinterpret_cast<unsigned long long *>(stage));
    // both end with a barrier; keys[] is sorted

    int32_t *order_f = order + (size_t)f * n_max;
    float *sorted_f = sorted5 + (size_t)f * 5 * n_pad;
    float4 *ysc_f = ysc ? ysc + (size_t)f * n_pad : nullptr;
    float *tsc_f = tsc ? tsc + (size_t)f * n_pad : nullptr;
    unsigned *ytile_f = ytile ? ytile + (size_t)f * (n_pad / kTile) : nullptr;
    if (STAGE) {
        // n_pad <= 4 * nth: at most four ranks per thread, r = tid + q * nth (a wavefront covers 64
        // consecutive ranks = one tile per q).
#pragma unroll
        for (int q = 0; q < 4; ++q) stage[e[q]] = mine[q];
        __syncthreads();
        float4 b[4];
        int idx[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int r = tid + q * nth;
            idx[q] = r < n_f ? (int)(unsigned)keys[r] : -1;
            b[q] = stage[idx[q] >= 0 ? idx[q] : 0];
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int r = tid + q * nth;
            if (r < n_pad) {  // uniform per wavefront (n_pad and nth are multiples of 64)
                bool regular = true;
                if (idx[q] >= 0)
                    regular = emit_ranked_box(b[q], idx[q], r, n_pad, order_f, sorted_f, ysc_f, tsc_f, m);
                else
                    emit_padding_row(r, n_pad, sorted_f, ysc_f, tsc_f);
                if (ytile_f != nullptr) {
                    const unsigned long long irregular = __ballot(!regular);
                    if (lane == 0) ytile_f[r / kTile] = irregular == 0 ? 1u : 0u;
                }
            }
        }
    } else {
        unsigned long long *kw = keys_ws + (size_t)f * n_pad + base;
        for (int i = tid; i < cnt; i += nth) kw[i] = keys[i];
        // the merge kernel scatters rows, so it can only clear tile flags: preset them here
        if (ytile_f != nullptr && chunk == 0)
            for (int t = tid; t < n_pad / kTile; t += nth) ytile_f[t] = 1u;
    }
    if (keep_preset != nullptr) {
        // fused path: every real box starts as a survivor, slots beyond the count are 0
        uint8_t *kp = keep_preset + (size_t)f * n_max;
        const int hi = (base + kSpan < n_max) ? base + kSpan : n_max;
        for (int i = base + tid; i < hi; i += nth) kp[i] = (i < n_f) ? 1 : 0;
    }
}

// Several chunks (of kMergeChunk boxes): the rank of a key is its position inside its own chunk
// plus the number of smaller keys in every other chunk (keys are unique, so ranks are too).
// The binary searches in the other chunks advance together, kMergeBatch chunks at a time, a
// fixed number of steps: the loads of one step do not depend on each other, so a thread waits
// for log2(chunk) + 1 round trips to memory however many chunks there are.  Four neighbouring
// lanes share an element (each takes every fourth chunk, the counts are summed across the four):
// a single large frame then fills the chip with workgroups instead of a quarter of it.
constexpr int kMergeChunk = 1024;
constexpr int kMergeBatch = 16;   // chunks searched together by the four lanes of an element
constexpr int kMergeLanes = 4;

__global__ void __launch_bounds__(256)
rank_merge_kernel(const float *__restrict__ boxes, const int32_t *__restrict__ counts, int n_max, int n_pad,
                  int n_chunks, const unsigned long long *__restrict__ keys_ws,
                  int32_t *__restrict__ order, float *__restrict__ sorted5,
                  float4 *__restrict__ ysc, unsigned *__restrict__ ytile, float *__restrict__ tsc, double m)
{
    constexpr int kMine = kMergeBatch / kMergeLanes;  // chunks of a batch per lane
    const int f = blockIdx.y;
    const int thread = blockIdx.x * blockDim.x + threadIdx.x;
    const int e = thread / kMergeLanes;   // n_pad is a multiple of 64: the four lanes of an element leave together
    const int q = thread % kMergeLanes;
    const int n_f = frame_count(counts, f, n_max);
    const unsigned long long *kw = keys_ws + (size_t)f * n_pad;
    if (e >= n_pad) return;
    float *sorted_f = sorted5 + (size_t)f * 5 * n_pad;
    float4 *ysc_f = ysc ? ysc + (size_t)f * n_pad : nullptr;
    float *tsc_f = tsc ? tsc + (size_t)f * n_pad : nullptr;
    if (e >= n_f) {
        if (q == 0) emit_padding_row(e, n_pad, sorted_f, ysc_f, tsc_f);
        return;
    }
    const unsigned long long key = kw[e];
    const int own = e / kMergeChunk;
    int rank = 0;
    for (int c0 = 0; c0 < n_chunks; c0 += kMergeBatch) {
        int below[kMine];  // keys of this lane's k-th chunk of the batch known to be smaller than `key`
        int cnt[kMine];
#pragma unroll
        for (int k = 0; k < kMine; ++k) {
            const int c = c0 + kMergeLanes * k + q;
            int left = n_f - c * kMergeChunk;
            left = left < 0 ? 0 : (left > kMergeChunk ? kMergeChunk : left);
            cnt[k] = (c < n_chunks && c != own) ? left : 0;
            below[k] = 0;
        }
        // below += step whenever the key `step` places further on is still smaller: no branches, and
        // a probe that would leave the chunk reads this thread's own key instead (never smaller)
#pragma unroll 1
        for (int step = kMergeChunk; step > 0; step >>= 1) {
            unsigned long long probe[kMine];
#pragma unroll
            for (int k = 0; k < kMine; ++k) {
                const int at = below[k] + step;
                probe[k] = kw[at <= cnt[k] ? (c0 + kMergeLanes * k + q) * kMergeChunk + at - 1 : e];
            }
#pragma unroll
            for (int k = 0; k < kMine; ++k) below[k] += probe[k] < key ? step : 0;
        }
#pragma unroll
        for (int k = 0; k < kMine; ++k) rank += below[k];
    }
    rank += __shfl_xor(rank, 1);
    rank += __shfl_xor(rank, 2);
    if (kMergeLanes > 4) rank += __shfl_xor(rank, 4);
    if (q != 0) return;
    rank += e - own * kMergeChunk;
    const int idx = (int)(unsigned)key;
    const bool regular = emit_ranked_box(reinterpret_cast<const float4 *>(boxes + (size_t)f * n_max * 4)[idx], idx, rank,
                                         n_pad, order + (size_t)f * n_max, sorted_f, ysc_f, tsc_f, m);
    // tile flags were preset to 1 by the chunk kernel; concurrent writers all store 0
    if (ytile != nullptr && !regular) ytile[(size_t)f * (n_pad / kTile) + rank / kTile] = 0u;
}
