// Part of nms_kernels.hip (included there, inside its anonymous namespace): the paper's rule with eliminated victims dropped from further tests, one workgroup per frame.
#pragma once

// ----------------------------------------------------------------------------- paper's rule, eliminated victims skipped

// Under the paper's rule a box survives iff NO better-ranked box eliminates it (section
// "Algorithm Correctness": V_i is the AND over all j), so a victim that has met one eliminator
// needs no further test -- it goes on eliminating others -- and most victims meet theirs among
// the best-ranked boxes.  One workgroup (16 wavefronts) handles a frame:
//
//   * all boxes of the frame are staged in LDS once (box and, per box, the value the decision
//     needs: its threshold T, or its area for the literal division);
//   * the victims still undecided are a LIST in LDS, in rank order (an entry is the byte offset
//     of the victim's box in the staged table);
//   * the outranking boxes ("candidates") are taken in stages [0,128), [128,256), [256,512) ...:
//     a stage's work is cut into items of (two candidate tiles = 128 boxes, one in each lane of
//     two register sets) x (32 consecutive list entries, read from LDS as broadcasts), dealt
//     round-robin to the wavefronts, so every wavefront has work in every stage however few
//     victims are left; the compare's lane mask != 0 is "this victim has an eliminator";
//   * after a stage the victims ranked before its end that are still alive are survivors, the
//     other alive ones are packed to the front of the list, and a table start[t] = number of
//     entries ranked before 64 t is rebuilt from the list (it tells each candidate group where
//     its victims begin, and where the victims begin that every lane of the group outranks).
//
// No pair is tested that involves a victim eliminated in an earlier stage; the result does not
// depend on the stage bounds, only the amount of work does.
//
// A frame is one compute unit's work, so this route is for batches of about as many frames as
// the chip has compute units or more.  Frames of at most NMS_SORT_CHUNK boxes.
constexpr int kEarlyWaves = 16;
constexpr int kEarlyThreads = kEarlyWaves * 64;
constexpr int kEarlyFirstStage = 128;                 // candidates of the first stage; each further stage doubles the bound
constexpr int kEarlyItemVictims = 32;                 // list entries of a work item (eight reads of four entries)
constexpr int kEarlyGroup = 2 * kTile;                // candidates of a work item: two tiles
constexpr int kEarlyTiles = NMS_SORT_CHUNK / kTile;   // 64

struct EarlyShared {
    float4 box[NMS_SORT_CHUNK];                    // rank order; y scaled by NMS_YSCALE in the y-scaled form
    float aux[NMS_SORT_CHUNK];                     // T, NMS_YSCALE * T, or the area
    int list[NMS_SORT_CHUNK + kEarlyItemVictims];  // undecided victims: 16 * rank, ascending; zeros behind the end
    uint8_t dead[NMS_SORT_CHUNK];                  // by list position: an eliminator was found in this stage
    int start[kEarlyTiles + 1];                    // start[t] = list entries ranked before 64 t
    int count[4 * kEarlyWaves];                    // packing: entries that go on, per 64 list positions
    int irregular;                                 // some y coordinate rules out the y-scaled form
};

template <int PAIR>
__device__ __forceinline__ bool early_hit(const float4 v, const float4 cb, float aux, float theta, float y_one)
{
    if (PAIR == kPairFastYScaled) return nms_eliminates_fast_yscaled(v.x, v.y, v.z, v.w, cb.x, cb.y, cb.z, cb.w, aux, y_one);
    if (PAIR == kPairFast) return nms_eliminates_fast(v.x, v.y, v.z, v.w, cb.x, cb.y, cb.z, cb.w, aux);
    return nms_eliminates_exact(v.x, v.y, v.z, v.w, cb.x, cb.y, cb.z, cb.w, aux, theta);
}

// Lanes 0 .. d-1 (the candidates of a tile that outrank a victim d ranks past the tile's first).
__device__ __forceinline__ unsigned long long early_below(int d)
{
    return d <= 0 ? 0ull : (d >= 64 ? ~0ull : (1ull << d) - 1ull);
}

// One work item: the list entries [32 jb, 32 jb + 32) against the candidates c_lo .. c_lo+127
// held in (cb0, aux0), (cb1, aux1).  DIAG: some of the victims are ranked within or before the
// group, so each compare mask is cut down to the candidates that outrank the victim (and to
// nothing for a second tile that does not exist).
template <int PAIR, bool DIAG>
__device__ __forceinline__ void early_item(EarlyShared &sh, int jb, int m, int c_lo, bool second, const float4 cb0,
                                           float aux0, const float4 cb1, float aux1, float theta, float y_one, int lane)
{
    const int4 *entries = reinterpret_cast<const int4 *>(sh.list + kEarlyItemVictims * jb);
    int4 e[kEarlyItemVictims / 4];
#pragma unroll
    for (int c = 0; c < kEarlyItemVictims / 4; ++c) e[c] = entries[c];  // same address in every lane: broadcasts
    unsigned word = 0;  // wave-uniform: bit k = entry 32 jb + k has an eliminator
#pragma unroll
    for (int c = 0; c < kEarlyItemVictims / 4; ++c) {
        const int off[4] = {e[c].x, e[c].y, e[c].z, e[c].w};
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float4 v = *reinterpret_cast<const float4 *>(reinterpret_cast<const char *>(sh.box) + off[u]);
            unsigned long long h0 = __ballot(early_hit<PAIR>(v, cb0, aux0, theta, y_one));
            unsigned long long h1 = __ballot(early_hit<PAIR>(v, cb1, aux1, theta, y_one));
            if (DIAG) {
                const int r = __builtin_amdgcn_readfirstlane(off[u]) >> 4;
                h0 &= early_below(r - c_lo);
                h1 &= second ? early_below(r - c_lo - kTile) : 0ull;
            }
            word |= ((h0 | h1) != 0ull ? 1u : 0u) << (4 * c + u);
        }
    }
    const int pos = kEarlyItemVictims * jb + lane;
    if (lane < kEarlyItemVictims && ((word >> lane) & 1u) != 0u && pos < m) sh.dead[pos] = 1;
}

// The stages of one frame; the table is staged, sh.list / sh.dead / sh.start describe the
// initial list (every rank) and keep_f is zero.
template <int PAIR>
__device__ __forceinline__ void early_exit_frame(EarlyShared &sh, int n_f, float theta, float y_one,
                                                 const int32_t *__restrict__ order_f, uint8_t *__restrict__ keep_f)
{
    const int tid = (int)threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int staged = (n_f + kTile - 1) / kTile * kTile;
    int m = n_f;  // list length
    int lo = 0;
    for (int bound = kEarlyFirstStage;; bound *= 2) {
        const int hi = bound < staged ? bound : staged;
        const bool last = hi >= n_f;
        const int groups = ((hi - lo) / kTile + 1) / 2;  // <= 32

        // lane = candidate group: where its victims begin, where those begin that all its lanes outrank, its items
        int p0 = 0, p1 = 0, items = 0;
        if (lane < groups) {
            const int t0 = lo / kTile + 2 * lane;
            p0 = sh.start[t0];
            p1 = sh.start[t0 + 2 < kEarlyTiles ? t0 + 2 : kEarlyTiles];
            items = (m + kEarlyItemVictims - 1) / kEarlyItemVictims - p0 / kEarlyItemVictims;
            items = p0 >= m ? 0 : items;
        }
        const int incl = (int)wave_inclusive_sum((unsigned)items);
        const int total = __builtin_amdgcn_readlane(incl, 63);
        int g_held = -1;
        float4 cb0 = make_float4(0.f, 0.f, 0.f, 0.f), cb1 = cb0;
        float aux0 = 0.f, aux1 = 0.f;
        for (int it = wave; it < total; it += kEarlyWaves) {
            const int g = __builtin_amdgcn_readfirstlane(__builtin_popcountll(__ballot(incl <= it)));
            const int jb = __builtin_amdgcn_readlane(p0, g) / kEarlyItemVictims + (it - __builtin_amdgcn_readlane(incl - items, g));
            const int p1_g = __builtin_amdgcn_readlane(p1, g);
            const int c_lo = lo + kEarlyGroup * g;
            const bool second = c_lo + kTile < hi;
            if (g != g_held) {
                cb0 = sh.box[c_lo + lane];
                aux0 = sh.aux[c_lo + lane];
                const int c1 = second ? c_lo + kTile + lane : lane;
                cb1 = sh.box[c1];
                aux1 = sh.aux[c1];
                g_held = g;
            }
            if (kEarlyItemVictims * jb < p1_g || !second)
                early_item<PAIR, true>(sh, jb, m, c_lo, second, cb0, aux0, cb1, aux1, theta, y_one, lane);
            else
                early_item<PAIR, false>(sh, jb, m, c_lo, second, cb0, aux0, cb1, aux1, theta, y_one, lane);
        }
        lds_barrier();

        // Entries still alive: those ranked before `hi` have met every better-ranked box and
        // survive; the others go on, packed to the front.  64 consecutive list positions report
        // how many go on in count[]; a prefix sum gives each its place.
        int entry[4];
        bool on[4];
        unsigned long long on_mask[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int i = tid + kEarlyThreads * j;
            const bool valid = i < m;
            entry[j] = valid ? sh.list[i] : 0;
            const bool alive = valid && sh.dead[valid ? i : 0] == 0;
            if (valid) sh.dead[i] = 0;
            const int r = entry[j] >> 4;
            if (alive && r < hi) keep_f[order_f[r]] = 1;
            on[j] = alive && r >= hi;
            on_mask[j] = __ballot(on[j]);
            if (lane == 0) sh.count[kEarlyWaves * j + wave] = __builtin_popcountll(on_mask[j]);
        }
        if (last) break;
        lds_barrier();
        const int mine = sh.count[lane];
        const int upto = (int)wave_inclusive_sum((unsigned)mine);
        const int m_new = __builtin_amdgcn_readlane(upto, 63);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int base = __builtin_amdgcn_readlane(upto - mine, kEarlyWaves * j + wave);
            if (on[j]) sh.list[base + __builtin_popcountll(on_mask[j] & ((1ull << lane) - 1ull))] = entry[j];
        }
        if (tid < kEarlyItemVictims) sh.list[m_new + tid] = 0;
        if (m_new == 0) break;
        lds_barrier();
        // start[t] = entries ranked before 64 t: entry i opens every tile after its predecessor's up to its own
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int i = tid + kEarlyThreads * j;
            if (i < m_new) {
                const int t_cur = sh.list[i] >> 10;
                const int t_prev = i > 0 ? sh.list[i - 1] >> 10 : -1;
                for (int t = t_prev + 1; t <= t_cur; ++t) sh.start[t] = i;
                if (i == m_new - 1)
                    for (int t = t_cur + 1; t <= kEarlyTiles; ++t) sh.start[t] = m_new;
            }
        }
        lds_barrier();
        m = m_new;
        lo = hi;
    }
}

// FAST: the division-free forms of nms_pair.h (the y-scaled one when every y coordinate of the
// frame allows it), else the literal division.
template <bool FAST>
__global__ void __launch_bounds__(kEarlyThreads)
early_exit_kernel(const float *__restrict__ sorted5, const int32_t *__restrict__ order,
                  const int32_t *__restrict__ counts, int n_max, int n_pad, NmsThetaConst th,
                  uint8_t *__restrict__ keep_out)
{
    __shared__ EarlyShared sh;
    const int f = blockIdx.x;
    const int tid = (int)threadIdx.x;
    const int n_f = frame_count(counts, f, n_max);
    const float *sorted_f = sorted5 + (size_t)f * 5 * n_pad;
    const float4 *box4 = reinterpret_cast<const float4 *>(sorted_f);
    const float *area = sorted_f + 4 * (size_t)n_pad;
    uint8_t *keep_f = keep_out + (size_t)f * n_max;
    const int32_t *order_f = order + (size_t)f * n_max;

    for (int i = tid; i < n_max; i += kEarlyThreads) keep_f[i] = 0;  // survivors are marked as they are found
    if (tid == 0) sh.irregular = 0;
    __syncthreads();  // also: the zero fill is complete before any survivor is marked
    const int staged = (n_f + kTile - 1) / kTile * kTile;  // padding rows of the table included
    bool irregular = false;
    for (int r = tid; r < staged; r += kEarlyThreads) {
        const float4 b = box4[r];
        sh.box[r] = b;
        sh.aux[r] = FAST ? nms_pair_threshold(area[r], th.m) : area[r];
        irregular |= !(nms_y_regular(b.y) && nms_y_regular(b.w));
    }
    if (FAST && irregular) sh.irregular = 1;
    for (int i = tid; i < NMS_SORT_CHUNK + kEarlyItemVictims; i += kEarlyThreads) sh.list[i] = i < n_f ? 16 * i : 0;
    reinterpret_cast<int *>(sh.dead)[tid] = 0;
    if (tid <= kEarlyTiles) sh.start[tid] = kTile * tid < n_f ? kTile * tid : n_f;
    lds_barrier();
    float y_one;  // NMS_YSCALE in a vector register (opaque to the compiler so it stays there)
    asm volatile("v_mov_b32 %0, 0x38800000" : "=v"(y_one));
    if (FAST && sh.irregular == 0) {
        for (int r = tid; r < staged; r += kEarlyThreads) {  // the rows this thread staged itself
            float4 b = sh.box[r];
            b.y *= NMS_YSCALE;
            b.w *= NMS_YSCALE;
            sh.box[r] = b;
            sh.aux[r] *= NMS_YSCALE;
        }
        lds_barrier();
        early_exit_frame<kPairFastYScaled>(sh, n_f, th.theta, y_one, order_f, keep_f);
    } else {
        early_exit_frame<FAST ? kPairFast : kPairExact>(sh, n_f, th.theta, y_one, order_f, keep_f);
    }
}
