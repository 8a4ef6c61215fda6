// Part of nms_kernels.hip (included there, inside its anonymous namespace): reduce step: row OR of the mask words.
#pragma once

// ----------------------------------------------------------------------------- reduce

// Lane = row.  Row tile tr owns tr + 1 words per row (the triangle), so a wavefront takes the
// tile rows p and T - 1 - p: T + 1 words of 512 contiguous bytes each, the same for every
// wavefront, all loads independent of each other (eight in flight per wavefront), no LDS and no
// barrier.  Each mask byte is read exactly once.  (Two rows per lane with 16-byte loads, and
// non-temporal loads, both measured slower.)
__global__ void __launch_bounds__(256)
reduce_rows_kernel(const unsigned long long *__restrict__ mask, const int32_t *__restrict__ order,
                   const int32_t *__restrict__ counts, int n_max, int n_pad, uint8_t *__restrict__ keep_out)
{
    const int f = blockIdx.y;
    const int lane = threadIdx.x & 63;
    const int T = n_pad / kTile;
    const int p = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 4 + (threadIdx.x >> 6)));
    if (p >= (T + 1) / 2) return;
    const int n_f = frame_count(counts, f, n_max);
    const unsigned long long *m = mask + (size_t)f * ((size_t)T * n_pad);
    uint8_t *keep_f = keep_out + (size_t)f * n_max;
    const int32_t *order_f = order + (size_t)f * n_max;
#pragma unroll 1
    for (int half = 0; half < 2; ++half) {
        const int tr = half == 0 ? p : T - 1 - p;
        if (half == 1 && tr == p) break;  // odd T: the middle tile row has no partner
        const int row = tr * kTile + lane;
        unsigned long long acc = 0;
        if (tr * kTile < n_f) {  // tile rows beyond the count are not written by the map step
            const unsigned long long *col = m + row;
#pragma unroll 8
            for (int w = 0; w <= tr; ++w) acc |= col[(size_t)w * n_pad];
        }
        if (row < n_f)
            keep_f[order_f[row]] = (acc == 0) ? 1 : 0;
        else if (row < n_max)
            keep_f[row] = 0;  // input slots beyond the frame's count
    }
}
