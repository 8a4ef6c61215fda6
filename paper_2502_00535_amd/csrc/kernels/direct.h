// Part of nms_kernels.hip (included there, inside its anonymous namespace): direct route: Algorithm 1 on the unsorted input with the score guard per pair, one launch.
#pragma once

// ----------------------------------------------------------------------------- direct (unranked) form

// The paper's own formulation for small frames: Algorithm 1 on the full n x n grid of
// the UNSORTED input with the score guard evaluated per pair, and Algorithm 2's row
// AND finished inside the workgroup, in one launch (no rank step, no mask, no scratch).
// It evaluates every unordered pair twice and pays two extra compares per pair for the
// guard, so it only wins where launch latency dominates: single frames up to a few
// thousand boxes.
//
// A workgroup owns ROWS consecutive victims (16, or fewer when that is needed to put a
// workgroup on every compute unit); its wavefronts split the n outranking
// candidates in 64-box tiles (lane = candidate c, victim r wave-uniform through scalar
// loads, exactly as in map_tile_kernel).  Each wavefront ends with one bit per victim,
// the workgroup ORs them through LDS and writes keep_out in input order.

// Which score compare decides "candidate c outranks victim r" for a whole tile:
// every candidate index below every victim index -> equal scores outrank (>=);
// every candidate index above -> strictly better only (>); the one tile that
// contains the victims themselves -> per lane.
enum { kGuardLowerIndex = 0, kGuardHigherIndex = 1, kGuardMixed = 2 };

// One victim row of the direct form: lane mask of the candidates that eliminate it.
template <bool FAST, int GUARD>
__device__ __forceinline__ unsigned long long direct_row(const float4 v, float v_score, int r, const float4 cb,
                                                         float c_score, float c_area, float c_T, int c,
                                                         const NmsThetaConst &th)
{
    bool hit;
    if (FAST)
        hit = nms_eliminates_fast(v.x, v.y, v.z, v.w, cb.x, cb.y, cb.z, cb.w, c_T);
    else
        hit = nms_eliminates_exact(v.x, v.y, v.z, v.w, cb.x, cb.y, cb.z, cb.w, c_area, th.theta);
    unsigned long long outranks;
    if (GUARD == kGuardLowerIndex) {
        outranks = __ballot(c_score >= v_score);
    } else if (GUARD == kGuardHigherIndex) {
        outranks = __ballot(c_score > v_score);
    } else {
        const unsigned long long lower = __ballot(c < r);
        outranks = (__ballot(c_score >= v_score) & lower) | (__ballot(c_score > v_score) & ~lower);
    }
    return __ballot(hit) & outranks;
}

template <bool FAST, int GUARD, bool CLAMP, int ROWS>
__device__ __forceinline__ unsigned direct_rows(const float4 *__restrict__ box4, const float *__restrict__ score,
                                                int v0, int n_f, const float4 cb, float c_score, float c_area, float c_T,
                                                int c, const NmsThetaConst &th)
{
    unsigned bits = 0;  // wave-uniform: bit k = victim v0+k is eliminated by a lane of this tile
    if (CLAMP) {
        // ragged last group of a frame: plain loop over the victims that exist
#pragma unroll 1
        for (int k = 0; k < ROWS && v0 + k < n_f; ++k) {
            const unsigned long long word = direct_row<FAST, GUARD>(box4[v0 + k], score[v0 + k], v0 + k, cb, c_score,
                                                                    c_area, c_T, c, th);
            bits |= (word != 0 ? 1u : 0u) << k;
        }
        return bits;
    }
    constexpr int kBatch = ROWS < 8 ? ROWS : 8;
#pragma unroll 1
    for (int half = 0; half < ROWS / kBatch; ++half) {
        // up to eight victims at a time: their scalar loads issue together, 40 SGPRs live
        float4 v[kBatch];
        float v_score[kBatch];
#pragma unroll
        for (int k = 0; k < kBatch; ++k) {
            v[k] = box4[v0 + kBatch * half + k];
            v_score[k] = score[v0 + kBatch * half + k];
        }
        unsigned half_bits = 0;
#pragma unroll
        for (int k = 0; k < kBatch; ++k) {
            const unsigned long long word = direct_row<FAST, GUARD>(v[k], v_score[k], v0 + kBatch * half + k, cb,
                                                                    c_score, c_area, c_T, c, th);
            half_bits |= (word != 0 ? 1u : 0u) << k;
        }
        bits |= half_bits << (kBatch * half);
    }
    return bits;
}

template <bool FAST, bool CLAMP, int ROWS>
__device__ __forceinline__ unsigned direct_tile(const float4 *__restrict__ box4, const float *__restrict__ score,
                                                int v0, int n_f, int t, const float4 cb, float c_score, float c_area,
                                                float c_T, int c, const NmsThetaConst &th)
{
    if (t * kTile + kTile - 1 < v0)
        return direct_rows<FAST, kGuardLowerIndex, CLAMP, ROWS>(box4, score, v0, n_f, cb, c_score, c_area, c_T, c, th);
    if (t * kTile > v0 + ROWS - 1)
        return direct_rows<FAST, kGuardHigherIndex, CLAMP, ROWS>(box4, score, v0, n_f, cb, c_score, c_area, c_T, c, th);
    return direct_rows<FAST, kGuardMixed, CLAMP, ROWS>(box4, score, v0, n_f, cb, c_score, c_area, c_T, c, th);
}

template <bool FAST, int ROWS>
__global__ void __launch_bounds__(1024)
direct_kernel(const float *__restrict__ boxes, const float *__restrict__ scores, const int32_t *__restrict__ counts,
              int n_max, NmsThetaConst th, uint8_t *__restrict__ keep_out)
{
    __shared__ unsigned hits[16];
    const int f = blockIdx.y;
    const int v0 = blockIdx.x * ROWS;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int n_waves = blockDim.x >> 6;
    const int n_f = frame_count(counts, f, n_max);
    uint8_t *keep_f = keep_out + (size_t)f * n_max;
    if (v0 >= n_f) {  // whole group beyond the frame's count (uniform for the workgroup)
        if (threadIdx.x < ROWS && v0 + (int)threadIdx.x < n_max) keep_f[v0 + threadIdx.x] = 0;
        return;
    }
    const float4 *box4 = reinterpret_cast<const float4 *>(boxes) + (size_t)f * n_max;
    const float *score = scores + (size_t)f * n_max;
    const int tiles = (n_f + kTile - 1) / kTile;
    const bool full = v0 + ROWS <= n_f;

    unsigned acc = 0;
    for (int t = wave; t < tiles; t += n_waves) {
        const int c = t * kTile + lane;
        const bool valid = c < n_f;
        const int cc = valid ? c : n_f - 1;
        const float4 cb = box4[cc];
        // a lane beyond the count never outranks anything: score -inf, index >= n_f
        const float c_score = valid ? score[cc] : -INFINITY;
        const float c_area = nms_box_area(cb.x, cb.y, cb.z, cb.w);
        const float c_T = FAST ? nms_pair_threshold(c_area, th.m) : 0.0f;
        if (full)
            acc |= direct_tile<FAST, false, ROWS>(box4, score, v0, n_f, t, cb, c_score, c_area, c_T, c, th);
        else
            acc |= direct_tile<FAST, true, ROWS>(box4, score, v0, n_f, t, cb, c_score, c_area, c_T, c, th);
    }
    if (lane == 0) hits[wave] = acc;
    __syncthreads();
    if (threadIdx.x < ROWS) {
        const int r = v0 + threadIdx.x;
        unsigned any = 0;
        for (int w = 0; w < n_waves; ++w) any |= hits[w];
        if (r < n_max) keep_f[r] = (r < n_f) ? (uint8_t)(((any >> threadIdx.x) & 1u) ^ 1u) : (uint8_t)0;
    }
}
