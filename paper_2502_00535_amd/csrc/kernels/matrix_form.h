// Part of nms_kernels.hip (included there, inside its anonymous namespace): the paper's byte-matrix layout and its k-partition reduce.
#pragma once

// ----------------------------------------------------------------------------- the paper's matrix form

// Algorithm 1 with the paper's own data layout: the boolean matrix B as capacity x capacity
// bytes over the unsorted input, one element per ordered pair (i, j), the score guard
// evaluated per pair.  A wavefront owns 256 consecutive columns j (four per lane, kept in
// registers) and kMatRows consecutive rows i (wave-uniform, scalar loads); each lane stores
// its four bytes of a row as one 32-bit word, 256 contiguous bytes per wavefront and row.
// Every byte is written, so the paper's memset of B is not needed.
constexpr int kMatRows = 16;

template <bool FAST>
__global__ void __launch_bounds__(256)
map_matrix_kernel(const float *__restrict__ boxes, const float *__restrict__ scores, int n, int cap,
                  NmsThetaConst th, uint8_t *__restrict__ B)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int j0 = blockIdx.x * 256 + 4 * lane;
    const int i0 = (blockIdx.y * 4 + wave) * kMatRows;
    if (i0 >= cap) return;
    const float4 *box4 = reinterpret_cast<const float4 *>(boxes);

    float4 cb[4];
    float c_score[4], c_area[4], c_T[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int c = j0 + q;
        const bool valid = c < n;
        cb[q] = valid ? box4[c] : make_float4(0.f, 0.f, 0.f, 0.f);
        c_score[q] = valid ? scores[c] : -INFINITY;  // an unused slot never outranks anything
        c_area[q] = nms_box_area(cb[q].x, cb[q].y, cb[q].z, cb[q].w);
        c_T[q] = FAST ? nms_pair_threshold(c_area[q], th.m) : 0.0f;
    }

    const int i_end = i0 + kMatRows < cap ? i0 + kMatRows : cap;
    for (int i = i0; i < i_end; ++i) {
        unsigned word = 0x01010101u;  // rows of unused slots: never guarded, stay 1
        if (i < n) {
            const float4 v = box4[i];
            const float v_score = scores[i];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                bool hit;
                if (FAST)
                    hit = nms_eliminates_fast(v.x, v.y, v.z, v.w, cb[q].x, cb[q].y, cb[q].z, cb[q].w, c_T[q]);
                else
                    hit = nms_eliminates_exact(v.x, v.y, v.z, v.w, cb[q].x, cb[q].y, cb[q].z, cb[q].w, c_area[q],
                                               th.theta);
                const bool outranks = c_score[q] > v_score || (c_score[q] == v_score && j0 + q < i);
                if (hit && outranks) word &= ~(1u << (8 * q));
            }
        }
        if (j0 < cap) *reinterpret_cast<unsigned *>(B + (size_t)i * cap + j0) = word;
    }
}

// Algorithm 2 as printed: one workgroup per row i with capacity / k threads; thread t
// looks at column t of each of the k partitions in turn, and a block-wide AND
// (__syncthreads_and: barrier plus wave ballots combined through LDS; CDNA has no barrier
// instruction that reduces) folds each partition into V_i.
__global__ void __launch_bounds__(1024)
reduce_matrix_kernel(const uint8_t *__restrict__ B, int cap, int k, uint8_t *__restrict__ V)
{
    const int i = blockIdx.x;
    const int part = cap / k;  // == blockDim.x
    size_t j = (size_t)i * cap + threadIdx.x;
    int v = __syncthreads_and(B[j]);
    for (int p = 1; p < k; ++p) {
        j += part;
        v = __syncthreads_and(v && B[j]);
    }
    if (threadIdx.x == 0) V[i] = (uint8_t)(v ? 1 : 0);
}
