// Part of nms_kernels.hip (included there, inside its anonymous namespace): classic greedy rule without a mask: one workgroup walks a frame in rank order (also with the variants).
#pragma once

// ----------------------------------------------------------------------------- greedy rule without a mask

// The classic sequential rule walked tile by tile in rank order, one workgroup (16
// wavefronts) per frame, no mask in memory.  Under this rule a box that is eliminated
// neither eliminates others nor needs any further test, so only the SURVIVORS are ever used
// as outranking boxes: about 600 of 4096 on frames like configuration 4, i.e. a seventh of
// the pair grid.  Worth it when a batch has about as many frames as the chip has compute
// units, since each frame is walked sequentially.
//
// A wavefront owns the tiles wave, wave + 16, wave + 32, wave + 48 and keeps their boxes in
// registers, lane = row; one wave-uniform 64-bit word per owned tile says which rows are
// eliminated (or do not exist).  For tile t = 0, 1, ...:
//   - its owner settles it: the rows still alive are visited in rank order; each one visited
//     is a survivor, is broadcast from its lane (v_readlane), eliminates the later rows of the
//     tile that it hits, and is appended to a list in LDS;
//   - barrier; every wavefront tests its later tiles against the list, one survivor at a
//     time (broadcast from the lane that read it from LDS), all 64 rows per instruction.
constexpr int kFusedWaves = 16;
constexpr int kFusedOwned = NMS_SORT_CHUNK / kTile / kFusedWaves;  // 4
constexpr long long kGreedyFusedBoxes = 128ll * 4096;  // nms_run_greedy_batched takes this route from frames * n_max boxes on

struct FusedCandidate {  // a survivor as an outranking box (fields a variant does not use are never read)
    float x1, y1, x2, y2, area, T, score;
    int label;
};

enum { kExTiesIgnore = 2, kExClasses = 4 };                       // flags of the variants (AUX)
enum { kExBoundary = 0, kExDivideGe = 1, kExDivideGt = 2 };      // how a variant decides the threshold (MODE)

// What the walk needs beyond the box table when it runs a variant of the rule (EX): see
// map_tile_ex_kernel below for the arithmetic.
struct FusedVariant {
    const float *ranked_score;    // [frames][n_pad], rank order (AUX)
    const int32_t *ranked_label;  // [frames][n_pad], rank order (AUX with labels)
    double boundary;              // rounding boundary of the division next to theta (MODE == kExBoundary)
    float offset;                 // 1 or 0
    int flags;
};

// Does candidate c eliminate the victim?  !EX: the default measure (MODE kExBoundary = the
// division-free form of nms_pair.h, else the literal division).  EX: the variants.
template <bool EX, bool IOU, int MODE, bool AUX>
__device__ __forceinline__ bool fused_hit(const float4 v, float v_area, float v_score, int v_label,
                                          const FusedCandidate &c, float theta, const FusedVariant &o)
{
    if (!EX) {
        if (MODE == kExBoundary) return nms_eliminates_fast(v.x, v.y, v.z, v.w, c.x1, c.y1, c.x2, c.y2, c.T);
        return nms_eliminates_exact(v.x, v.y, v.z, v.w, c.x1, c.y1, c.x2, c.y2, c.area, theta);
    }
    const float iw = fmaxf(0.0f, (fminf(v.z, c.x2) - fmaxf(v.x, c.x1)) + o.offset);
    const float ih = fmaxf(0.0f, (fminf(v.w, c.y2) - fmaxf(v.y, c.y1)) + o.offset);
    const float inter = iw * ih;
    const float denom = IOU ? (v_area + c.area) - inter : c.area;
    bool hit;
    if (MODE == kExBoundary && !IOU)
        hit = inter >= c.T;
    else if (MODE == kExBoundary)
        hit = (double)inter >= o.boundary * (double)denom;
    else if (MODE == kExDivideGe)
        hit = !(inter / denom < theta);
    else
        hit = inter / denom > theta;
    if (AUX) {
        hit = hit && ((o.flags & kExTiesIgnore) == 0 || c.score > v_score);
        hit = hit && ((o.flags & kExClasses) == 0 || c.label == v_label);
    }
    return hit;
}

// Lane `src` (wave-uniform) of a per-lane candidate, as a wave-uniform value.
__device__ __forceinline__ FusedCandidate broadcast_candidate(const FusedCandidate &mine, int src)
{
    FusedCandidate c;
    c.x1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, mine.x1), src));
    c.y1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, mine.y1), src));
    c.x2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, mine.x2), src));
    c.y2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, mine.y2), src));
    c.area = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, mine.area), src));
    c.T = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, mine.T), src));
    c.score = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, mine.score), src));
    c.label = __builtin_amdgcn_readlane(mine.label, src);
    return c;
}

template <bool EX, bool IOU, int MODE, bool AUX>
__global__ void __launch_bounds__(kFusedWaves * 64)
greedy_fused_kernel(const float *__restrict__ sorted5, const int32_t *__restrict__ order,
                    const int32_t *__restrict__ counts, int n_max, int n_pad, NmsThetaConst th, FusedVariant opt,
                    uint8_t *__restrict__ keep_out)
{
    __shared__ FusedCandidate list_s[2][kTile];  // survivors of tile t in buffer t & 1
    __shared__ int count_s[2];
    const int f = blockIdx.x;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int n_f = frame_count(counts, f, n_max);
    const int tiles_f = (n_f + kTile - 1) / kTile;
    const float *sorted_f = sorted5 + (size_t)f * 5 * n_pad;
    const float4 *box4 = reinterpret_cast<const float4 *>(sorted_f);
    const float *area = sorted_f + 4 * (size_t)n_pad;
    uint8_t *keep_f = keep_out + (size_t)f * n_max;
    const int32_t *order_f = order + (size_t)f * n_max;

    // the owned tiles: boxes (also in their role as outranking boxes) and the rows that are out
    float4 vb[kFusedOwned];
    FusedCandidate self[kFusedOwned];
    unsigned long long out[kFusedOwned];  // wave-uniform; bit r: row r is eliminated, settled or does not exist
#pragma unroll
    for (int i = 0; i < kFusedOwned; ++i) {
        const int tr = wave + kFusedWaves * i;
        const bool has = tr < tiles_f;
        const int r = has ? tr * kTile + lane : 0;  // rows of a partial last tile beyond n_f are padding rows of the table
        vb[i] = box4[r];
        FusedCandidate me;
        me.x1 = vb[i].x, me.y1 = vb[i].y, me.x2 = vb[i].z, me.y2 = vb[i].w;
        me.area = EX ? ((vb[i].z - vb[i].x) + opt.offset) * ((vb[i].w - vb[i].y) + opt.offset) : area[r];
        me.T = MODE == kExBoundary ? nms_pair_threshold(me.area, EX ? opt.boundary : th.m) : 0.0f;
        me.score = AUX ? opt.ranked_score[(size_t)f * n_pad + r] : 0.0f;
        me.label = (AUX && (opt.flags & kExClasses)) ? opt.ranked_label[(size_t)f * n_pad + r] : 0;
        self[i] = me;
        const int first = tr * kTile;
        out[i] = !has ? ~0ull : (first + kTile <= n_f ? 0ull : ~0ull << (n_f - first));
    }

    for (int t = 0; t < tiles_f; ++t) {
        const int buf = t & 1;
        if (wave == (t & (kFusedWaves - 1))) {
            // settle tile t = owned tile number t / 16
            float4 v = vb[0];
            FusedCandidate mine = self[0];
            unsigned long long todo = ~out[0];
#pragma unroll
            for (int i = 1; i < kFusedOwned; ++i) {
                if ((t >> 4) == i) {  // wave-uniform
                    v = vb[i];
                    mine = self[i];
                    todo = ~out[i];
                }
            }
            unsigned long long kept = 0;
            int count = 0;
            while (todo != 0) {
                const int c = (int)__builtin_ctzll(todo);  // best-ranked row still alive: a survivor
                todo &= todo - 1ull;
                kept |= 1ull << c;
                const FusedCandidate cand = broadcast_candidate(mine, c);
                const bool hit = fused_hit<EX, IOU, MODE, AUX>(v, mine.area, mine.score, mine.label, cand, th.theta, opt) &&
                                 lane > c;
                todo &= ~__ballot(hit);
                if (lane == 0) list_s[buf][count] = cand;
                ++count;
            }
            if (lane == 0) count_s[buf] = count;
            const int r = t * kTile + lane;
            if (r < n_f) keep_f[order_f[r]] = (uint8_t)((kept >> lane) & 1ull);
#pragma unroll
            for (int i = 0; i < kFusedOwned; ++i)
                if ((t >> 4) == i) out[i] = ~0ull;
        }
        lds_barrier();
        // the survivors of tile t against the later owned tiles that still have a row alive
        const int count = __builtin_amdgcn_readfirstlane(count_s[buf]);
        bool any = false;
#pragma unroll
        for (int i = 0; i < kFusedOwned; ++i) any = any || (wave + kFusedWaves * i > t && out[i] != ~0ull);
        if (count > 0 && any) {
            const FusedCandidate held = list_s[buf][lane < count ? lane : 0];  // lane k holds survivor k
            for (int k = 0; k < count; ++k) {
                const FusedCandidate cand = broadcast_candidate(held, k);
#pragma unroll
                for (int i = 0; i < kFusedOwned; ++i) {
                    if (wave + kFusedWaves * i > t && out[i] != ~0ull)  // wave-uniform
                        out[i] |= __ballot(fused_hit<EX, IOU, MODE, AUX>(vb[i], self[i].area, self[i].score, self[i].label,
                                                                          cand, th.theta, opt));
                }
            }
        }
    }
    for (int i = n_f + (int)threadIdx.x; i < n_max; i += blockDim.x) keep_f[i] = 0;  // slots beyond the count
}
