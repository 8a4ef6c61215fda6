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

// Algorithm 2's result on the byte matrix, V_i = AND over j of B_ij (ReduceKernel
// postcondition), with its partition count k as the knob the paper sweeps: the row is cut in
// k partitions of cap / k columns and a row is given (cap / k) / VEC lanes; lane t folds column
// group t of every partition in turn, k loads that do not depend on each other (issued
// four at a time), VEC = 8 bytes per load when a partition is a multiple of eight columns
// (one 64-bit load, "some byte is zero" decided with integer arithmetic), else byte loads.
// A row of at most 64 lanes is one wavefront and ends in a single ballot; wider rows take
// several wavefronts of one workgroup, which meet once in LDS.  Small k: many lanes, few
// loads each; large k: few lanes, long chains -- the same trade the paper's threads-per-block
// sweep makes, without a workgroup-wide barrier per partition.
__device__ __forceinline__ bool has_zero_byte(unsigned long long w)
{
    return ((w - 0x0101010101010101ull) & ~w & 0x8080808080808080ull) != 0ull;
}

template <int VEC>
__global__ void __launch_bounds__(1024)
reduce_matrix_kernel(const uint8_t *__restrict__ B, int cap, int k, int waves_per_row, uint8_t *__restrict__ V)
{
    __shared__ unsigned zero_seen[16];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int rows_per_block = (int)(blockDim.x >> 6) / waves_per_row;
    const int row_in_block = wave / waves_per_row;
    const int sub = wave - row_in_block * waves_per_row;  // which wavefront of its row
    const int i = blockIdx.x * rows_per_block + row_in_block;
    const int part = cap / k;
    const int col = (sub * 64 + lane) * VEC;              // first column of this lane's group inside a partition
    const bool active = row_in_block < rows_per_block && i < cap && col < part;
    bool zero = false;
    if (active) {
        const uint8_t *row = B + (size_t)i * cap + col;
        int p = 0;
        for (; p + 4 <= k; p += 4) {
            if (VEC == 8) {
                const unsigned long long a = *reinterpret_cast<const unsigned long long *>(row + (size_t)p * part);
                const unsigned long long b = *reinterpret_cast<const unsigned long long *>(row + (size_t)(p + 1) * part);
                const unsigned long long c = *reinterpret_cast<const unsigned long long *>(row + (size_t)(p + 2) * part);
                const unsigned long long d = *reinterpret_cast<const unsigned long long *>(row + (size_t)(p + 3) * part);
                zero |= has_zero_byte(a) | has_zero_byte(b) | has_zero_byte(c) | has_zero_byte(d);
            } else {
                const uint8_t a = row[(size_t)p * part], b = row[(size_t)(p + 1) * part];
                const uint8_t c = row[(size_t)(p + 2) * part], d = row[(size_t)(p + 3) * part];
                zero |= (a == 0) | (b == 0) | (c == 0) | (d == 0);
            }
        }
        for (; p < k; ++p) {
            if (VEC == 8)
                zero |= has_zero_byte(*reinterpret_cast<const unsigned long long *>(row + (size_t)p * part));
            else
                zero |= row[(size_t)p * part] == 0;
        }
    }
    const bool wave_zero = __ballot(zero) != 0ull;
    if (waves_per_row == 1) {
        if (lane == 0 && active) V[i] = wave_zero ? 0 : 1;  // lane 0's column 0 exists whenever the row does
        return;
    }
    if (lane == 0) zero_seen[wave] = wave_zero ? 1u : 0u;
    __syncthreads();
    if (sub == 0 && lane == 0 && row_in_block < rows_per_block && i < cap) {
        unsigned any = 0;
        for (int w = 0; w < waves_per_row; ++w) any |= zero_seen[wave + w];
        V[i] = any ? 0 : 1;
    }
}
