// VALU issue-rate probe for gfx950: lane-operations per second of single instructions,
// measured with 8 wavefronts per SIMD on every CU and eight independent dependency chains
// per lane.  Used to derive the ALU ceiling of the NMS pair test from measurement instead
// of from the data sheet alone.  Stand-alone program: `python -m paper_2502_00535_amd.build
// --probe` builds it as paper_2502_00535_amd/valu_probe; run it on the GPU with no arguments.
// Only VALU instructions without side effects on SCC/EXEC are probed (inline asm that
// touched SCC could corrupt the loop branch).
#include <hip/hip_runtime.h>
#include <cstdio>
#include <vector>
#include <string>

#define CHECK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %s:%d\n", hipGetErrorString(e), __FILE__, __LINE__); return 1; } } while (0)

#define BODY(INSTR) \
    float x0 = threadIdx.x, x1 = x0 + 1, x2 = x0 + 2, x3 = x0 + 3, x4 = x0 + 4, x5 = x0 + 5, x6 = x0 + 6, x7 = x0 + 7; \
    for (int i = 0; i < iters; ++i) { \
        _Pragma("unroll") for (int u = 0; u < 8; ++u) { \
            asm volatile(INSTR : "+v"(x0) : "v"(a), "s"(sb) : "vcc", "s20", "s21", "s22", "s23"); asm volatile(INSTR : "+v"(x1) : "v"(a), "s"(sb) : "vcc", "s20", "s21", "s22", "s23"); \
            asm volatile(INSTR : "+v"(x2) : "v"(a), "s"(sb) : "vcc", "s20", "s21", "s22", "s23"); asm volatile(INSTR : "+v"(x3) : "v"(a), "s"(sb) : "vcc", "s20", "s21", "s22", "s23"); \
            asm volatile(INSTR : "+v"(x4) : "v"(a), "s"(sb) : "vcc", "s20", "s21", "s22", "s23"); asm volatile(INSTR : "+v"(x5) : "v"(a), "s"(sb) : "vcc", "s20", "s21", "s22", "s23"); \
            asm volatile(INSTR : "+v"(x6) : "v"(a), "s"(sb) : "vcc", "s20", "s21", "s22", "s23"); asm volatile(INSTR : "+v"(x7) : "v"(a), "s"(sb) : "vcc", "s20", "s21", "s22", "s23"); \
        } \
    } \
    out[blockIdx.x * blockDim.x + threadIdx.x] = x0 + x1 + x2 + x3 + x4 + x5 + x6 + x7;

__global__ void k_add(float *out, float a, float sb, int iters) { BODY("v_add_f32 %0, %1, %0") }
__global__ void k_add_s(float *out, float a, float sb, int iters) { BODY("v_add_f32 %0, %2, %0") }
__global__ void k_min(float *out, float a, float sb, int iters) { BODY("v_min_f32 %0, %1, %0") }
__global__ void k_min_s(float *out, float a, float sb, int iters) { BODY("v_min_f32 %0, %2, %0") }
__global__ void k_max(float *out, float a, float sb, int iters) { BODY("v_max_f32 %0, %1, %0") }
__global__ void k_mul(float *out, float a, float sb, int iters) { BODY("v_mul_f32 %0, %1, %0") }
__global__ void k_sub(float *out, float a, float sb, int iters) { BODY("v_sub_f32 %0, %1, %0") }
__global__ void k_fma(float *out, float a, float sb, int iters) { BODY("v_fma_f32 %0, %1, %0, %0") }
__global__ void k_fmac(float *out, float a, float sb, int iters) { BODY("v_fmac_f32 %0, %1, %1") }
__global__ void k_cmp(float *out, float a, float sb, int iters) { BODY("v_cmp_ge_f32 vcc, %1, %0") }
__global__ void k_cmp64(float *out, float a, float sb, int iters) { BODY("v_cmp_ge_f32 s[20:21], %1, %0") }
__global__ void k_mov(float *out, float a, float sb, int iters) { BODY("v_mov_b32 %0, %1") }
__global__ void k_and(float *out, float a, float sb, int iters) { BODY("v_and_b32 %0, %1, %0") }
__global__ void k_max3(float *out, float a, float sb, int iters) { BODY("v_max3_f32 %0, %1, %0, %0") }
__global__ void k_pkadd(float *out, float a, float sb, int iters) { BODY("v_add_u32 %0, %1, %0") }
__global__ void k_mini(float *out, float a, float sb, int iters) { BODY("v_min_i32 %0, %1, %0") }
__global__ void k_maxu(float *out, float a, float sb, int iters) { BODY("v_max_u32 %0, %1, %0") }
__global__ void k_addc(float *out, float a, float sb, int iters) { BODY("v_add_f32 %0, 1.0, %0") }
__global__ void k_andor(float *out, float a, float sb, int iters) { BODY("v_and_or_b32 %0, %1, %0, %0") }
__global__ void k_fma3(float *out, float a, float sb, int iters) { BODY("v_fma_f32 %0, %1, %1, %0") }
__global__ void k_mulabs(float *out, float a, float sb, int iters) { BODY("v_mul_f32_e64 %0, %1, |%0|") }
__global__ void k_cnd(float *out, float a, float sb, int iters) { BODY("v_cndmask_b32 %0, %1, %0, vcc") }
__global__ void k_addclamp(float *out, float a, float sb, int iters) { BODY("v_add_f32_e64 %0, 1.0, %0 clamp") }
__global__ void k_subclamp(float *out, float a, float sb, int iters) { BODY("v_sub_f32_e64 %0, %1, %0 clamp") }
__global__ void k_rcp(float *out, float a, float sb, int iters) { BODY("v_rcp_f32 %0, %0") }
__global__ void k_fmaclamp(float *out, float a, float sb, int iters) { BODY("v_fma_f32 %0, %0, %1, %1 clamp") }
__global__ void k_fmaxaa(float *out, float a, float sb, int iters) { BODY("v_fma_f32 %0, %0, %1, %1") }
__global__ void k_fmaaxa(float *out, float a, float sb, int iters) { BODY("v_fma_f32 %0, %1, %0, %1") }
__global__ void k_fmaxa1(float *out, float a, float sb, int iters) { BODY("v_fma_f32 %0, %0, %1, 1.0") }
__global__ void k_madxa(float *out, float a, float sb, int iters) { BODY("v_fma_f32 %0, %1, %0, 1.0 clamp") }

// float64 instructions (the variants' exact threshold compare uses a convert, a multiply and a compare)
#define BODYD(INSTR) \
    double x0 = threadIdx.x, x1 = x0 + 1, x2 = x0 + 2, x3 = x0 + 3, x4 = x0 + 4, x5 = x0 + 5, x6 = x0 + 6, x7 = x0 + 7; \
    const double ad = a; \
    for (int i = 0; i < iters; ++i) { \
        _Pragma("unroll") for (int u = 0; u < 8; ++u) { \
            asm volatile(INSTR : "+v"(x0) : "v"(ad), "v"(a) : "vcc"); asm volatile(INSTR : "+v"(x1) : "v"(ad), "v"(a) : "vcc"); \
            asm volatile(INSTR : "+v"(x2) : "v"(ad), "v"(a) : "vcc"); asm volatile(INSTR : "+v"(x3) : "v"(ad), "v"(a) : "vcc"); \
            asm volatile(INSTR : "+v"(x4) : "v"(ad), "v"(a) : "vcc"); asm volatile(INSTR : "+v"(x5) : "v"(ad), "v"(a) : "vcc"); \
            asm volatile(INSTR : "+v"(x6) : "v"(ad), "v"(a) : "vcc"); asm volatile(INSTR : "+v"(x7) : "v"(ad), "v"(a) : "vcc"); \
        } \
    } \
    out[blockIdx.x * blockDim.x + threadIdx.x] = (float)(x0 + x1 + x2 + x3 + x4 + x5 + x6 + x7);

__global__ void k_mul64(float *out, float a, float sb, int iters) { BODYD("v_mul_f64 %0, %1, %0") }
__global__ void k_fma64(float *out, float a, float sb, int iters) { BODYD("v_fma_f64 %0, %1, %0, %0") }
__global__ void k_cmpf64(float *out, float a, float sb, int iters) { BODYD("v_cmp_ge_f64 vcc, %1, %0") }
__global__ void k_cvt64(float *out, float a, float sb, int iters) { BODYD("v_cvt_f64_f32 %0, %2") }

typedef void (*kern_t)(float *, float, float, int);

int main()
{
    hipDeviceProp_t prop;
    CHECK(hipGetDeviceProperties(&prop, 0));
    printf("device %s, CUs %d, clock %d kHz\n", prop.name, prop.multiProcessorCount, prop.clockRate);
    const int blocks = prop.multiProcessorCount * 8, threads = 256;  // 8 waves per SIMD
    float *out;
    CHECK(hipMalloc(&out, sizeof(float) * blocks * threads));
    struct Item { const char *name; kern_t k; int per; };
    std::vector<Item> items = {
        {"v_add_f32 vv", k_add, 1}, {"v_add_f32 sv", k_add_s, 1}, {"v_min_f32 vv", k_min, 1}, {"v_min_f32 sv", k_min_s, 1},
        {"v_max_f32", k_max, 1}, {"v_mul_f32", k_mul, 1}, {"v_sub_f32", k_sub, 1}, {"v_fma_f32", k_fma, 1}, {"v_fmac_f32", k_fmac, 1},
        {"v_cmp vcc", k_cmp, 1}, {"v_cmp sgpr", k_cmp64, 1}, {"v_mov_b32", k_mov, 1}, {"v_and_b32", k_and, 1}, {"v_max3_f32", k_max3, 1},
        {"v_add_u32", k_pkadd, 1}, {"v_rcp_f32", k_rcp, 1}, {"v_min_i32", k_mini, 1}, {"v_max_u32", k_maxu, 1}, {"v_add_f32 1.0", k_addc, 1}, {"v_and_or_b32", k_andor, 1}, {"v_fma_f32 3src", k_fma3, 1}, {"v_mul_f32 |abs|", k_mulabs, 1}, {"v_cndmask", k_cnd, 1}, {"v_add_f32 clamp", k_addclamp, 1}, {"v_sub_f32 clamp", k_subclamp, 1}, {"v_fma_f32 x,a,a clamp", k_fmaclamp, 1}, {"v_fma_f32 x,a,a", k_fmaxaa, 1}, {"v_fma_f32 a,x,a", k_fmaaxa, 1}, {"v_fma_f32 x,a,1.0", k_fmaxa1, 1}, {"v_fma_f32 a,x,1.0 clamp", k_madxa, 1},
        {"v_mul_f64", k_mul64, 1}, {"v_fma_f64", k_fma64, 1}, {"v_cmp_ge_f64", k_cmpf64, 1}, {"v_cvt_f64_f32", k_cvt64, 1},
    };
    const int iters = 2000;
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    for (auto &it : items) {
        it.k<<<blocks, threads>>>(out, 1.5f, 0.25f, 10);
        CHECK(hipDeviceSynchronize());
        CHECK(hipEventRecord(e0));
        it.k<<<blocks, threads>>>(out, 1.5f, 0.25f, iters);
        CHECK(hipEventRecord(e1));
        CHECK(hipEventSynchronize(e1));
        float ms;
        CHECK(hipEventElapsedTime(&ms, e0, e1));
        double instr = (double)blocks * threads * iters * 64.0;  // lane-instructions of the probed kind (64 per loop trip per lane)
        printf("%-16s %8.3f ms  %7.2f T lane-ops/s (x%d VALU per slot)\n", it.name, ms, instr * 1.0 / (ms * 1e-3) / 1e12, it.per);
        fflush(stdout);
    }
    return 0;
}
