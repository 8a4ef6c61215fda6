// Measurement kernels of bench.py (not part of the NMS library): issue rate of single VALU
// instructions on the whole chip, and the shader clock under that load.
//
// The pair test of the NMS map kernel is ten VALU instructions per 64 pairs and nothing else
// that matters, so its ceiling is the rate at which a SIMD issues those instructions.  The
// published FP32 vector peak counts a fused multiply-add per lane per cycle on 32 lanes; min,
// max and compare issue at half that lane rate, and none of the ten is a multiply-add.  bench.py
// measures the rates in the run that reports them instead of trusting constants.
//
// Each probe: 8 wavefronts per SIMD on every compute unit, eight independent dependency chains
// per lane, `iters` loop trips of 64 instructions of the probed kind.  Only VALU instructions
// without side effects on SCC/EXEC are probed.  One wavefront also samples the shader-clock
// counter and the constant-rate wall clock at its start and end.
#include <hip/hip_runtime.h>

#include <stdint.h>

namespace {

#define PROBE_BODY(INSTR)                                                                                       \
    unsigned long long c0 = 0, w0 = 0;                                                                          \
    const bool sampler = clocks != nullptr && blockIdx.x == 0 && threadIdx.x == 0;                              \
    if (sampler) { c0 = clock64(); w0 = wall_clock64(); }                                                       \
    float x0 = threadIdx.x, x1 = x0 + 1, x2 = x0 + 2, x3 = x0 + 3, x4 = x0 + 4, x5 = x0 + 5, x6 = x0 + 6,       \
          x7 = x0 + 7;                                                                                          \
    for (int i = 0; i < iters; ++i) {                                                                           \
        _Pragma("unroll") for (int u = 0; u < 8; ++u) {                                                         \
            asm volatile(INSTR : "+v"(x0) : "v"(a), "s"(sb) : "vcc", "s20", "s21");                             \
            asm volatile(INSTR : "+v"(x1) : "v"(a), "s"(sb) : "vcc", "s20", "s21");                             \
            asm volatile(INSTR : "+v"(x2) : "v"(a), "s"(sb) : "vcc", "s20", "s21");                             \
            asm volatile(INSTR : "+v"(x3) : "v"(a), "s"(sb) : "vcc", "s20", "s21");                             \
            asm volatile(INSTR : "+v"(x4) : "v"(a), "s"(sb) : "vcc", "s20", "s21");                             \
            asm volatile(INSTR : "+v"(x5) : "v"(a), "s"(sb) : "vcc", "s20", "s21");                             \
            asm volatile(INSTR : "+v"(x6) : "v"(a), "s"(sb) : "vcc", "s20", "s21");                             \
            asm volatile(INSTR : "+v"(x7) : "v"(a), "s"(sb) : "vcc", "s20", "s21");                             \
        }                                                                                                       \
    }                                                                                                           \
    out[blockIdx.x * blockDim.x + threadIdx.x] = x0 + x1 + x2 + x3 + x4 + x5 + x6 + x7;                         \
    if (sampler) {                                                                                              \
        clocks[0] = clock64() - c0;                                                                             \
        clocks[1] = wall_clock64() - w0;                                                                        \
    }

#define PROBE(NAME, INSTR) \
    __global__ void NAME(float *out, unsigned long long *clocks, float a, float sb, int iters) { PROBE_BODY(INSTR) }

// the ten instructions of the pair test, in the operand forms the map kernel uses
PROBE(p_sub_vv, "v_sub_f32 %0, %1, %0")
PROBE(p_add_const, "v_add_f32 %0, 1.0, %0")
PROBE(p_add_clamp, "v_add_f32_e64 %0, %1, %0 clamp")
PROBE(p_mul_vv, "v_mul_f32 %0, %1, %0")
PROBE(p_min_sv, "v_min_f32 %0, %2, %0")
PROBE(p_max_sv, "v_max_f32 %0, %2, %0")
PROBE(p_cmp_sgpr, "v_cmp_ge_f32 s[20:21], %1, %0")
// for the table of issue classes
PROBE(p_add_vv, "v_add_f32 %0, %1, %0")
PROBE(p_add_sv, "v_add_f32 %0, %2, %0")
PROBE(p_min_vv, "v_min_f32 %0, %1, %0")
PROBE(p_max_vv, "v_max_f32 %0, %1, %0")
PROBE(p_cmp_vcc, "v_cmp_ge_f32 vcc, %1, %0")
PROBE(p_mov, "v_mov_b32 %0, %1")
PROBE(p_fma, "v_fma_f32 %0, %1, %0, %0")
PROBE(p_fma_const, "v_fma_f32 %0, %0, %1, 1.0")
PROBE(p_fmac, "v_fmac_f32 %0, %1, %1")
PROBE(p_max3, "v_max3_f32 %0, %1, %0, %0")
PROBE(p_min_i32, "v_min_i32 %0, %1, %0")
PROBE(p_max_u32, "v_max_u32 %0, %1, %0")
PROBE(p_and, "v_and_b32 %0, %1, %0")
PROBE(p_add_u32, "v_add_u32 %0, %1, %0")
PROBE(p_mul_abs, "v_mul_f32_e64 %0, %1, |%0|")
PROBE(p_sub_clamp, "v_sub_f32_e64 %0, %1, %0 clamp")
PROBE(p_mul_clamp, "v_mul_f32_e64 %0, %1, %0 clamp")
PROBE(p_rcp, "v_rcp_f32 %0, %0")
PROBE(p_readlane, "v_readlane_b32 s20, %0, 5")
PROBE(p_cmp_lt_u32, "v_cmp_lt_u32 vcc, %1, %0")

// float64 instructions (the variants' exact threshold compare uses a convert, a multiply and a compare)
#define PROBE_BODY_F64(INSTR)                                                                                   \
    unsigned long long c0 = 0, w0 = 0;                                                                          \
    const bool sampler = clocks != nullptr && blockIdx.x == 0 && threadIdx.x == 0;                              \
    if (sampler) { c0 = clock64(); w0 = wall_clock64(); }                                                       \
    double x0 = threadIdx.x, x1 = x0 + 1, x2 = x0 + 2, x3 = x0 + 3, x4 = x0 + 4, x5 = x0 + 5, x6 = x0 + 6,      \
           x7 = x0 + 7;                                                                                         \
    const double ad = a;                                                                                        \
    for (int i = 0; i < iters; ++i) {                                                                           \
        _Pragma("unroll") for (int u = 0; u < 8; ++u) {                                                         \
            asm volatile(INSTR : "+v"(x0) : "v"(ad), "v"(a) : "vcc");                                           \
            asm volatile(INSTR : "+v"(x1) : "v"(ad), "v"(a) : "vcc");                                           \
            asm volatile(INSTR : "+v"(x2) : "v"(ad), "v"(a) : "vcc");                                           \
            asm volatile(INSTR : "+v"(x3) : "v"(ad), "v"(a) : "vcc");                                           \
            asm volatile(INSTR : "+v"(x4) : "v"(ad), "v"(a) : "vcc");                                           \
            asm volatile(INSTR : "+v"(x5) : "v"(ad), "v"(a) : "vcc");                                           \
            asm volatile(INSTR : "+v"(x6) : "v"(ad), "v"(a) : "vcc");                                           \
            asm volatile(INSTR : "+v"(x7) : "v"(ad), "v"(a) : "vcc");                                           \
        }                                                                                                       \
    }                                                                                                           \
    out[blockIdx.x * blockDim.x + threadIdx.x] = (float)(x0 + x1 + x2 + x3 + x4 + x5 + x6 + x7);             \
    if (sampler) {                                                                                              \
        clocks[0] = clock64() - c0;                                                                             \
        clocks[1] = wall_clock64() - w0;                                                                        \
    }

#define PROBE_F64(NAME, INSTR) \
    __global__ void NAME(float *out, unsigned long long *clocks, float a, float sb, int iters) { PROBE_BODY_F64(INSTR) }

PROBE_F64(p_mul_f64, "v_mul_f64 %0, %1, %0")
PROBE_F64(p_fma_f64, "v_fma_f64 %0, %1, %0, %0")
PROBE_F64(p_cmp_f64, "v_cmp_ge_f64 vcc, %1, %0")
PROBE_F64(p_cvt_f64_f32, "v_cvt_f64_f32 %0, %2")
PROBE_F64(p_cmp_lt_u64, "v_cmp_lt_u64 vcc, %1, %0")

// The pair test's ten instructions as the fused map kernel issues them (victim coordinates as
// scalar operands), on eight chains per lane, nothing else in the loop: the ceiling of that mix.
#define ON_ALL_CHAINS(INSTR)                                                                                     \
    asm volatile(INSTR : "+v"(x0) : "v"(a), "s"(sb) : "s20", "s21"); asm volatile(INSTR : "+v"(x1) : "v"(a), "s"(sb) : "s20", "s21"); \
    asm volatile(INSTR : "+v"(x2) : "v"(a), "s"(sb) : "s20", "s21"); asm volatile(INSTR : "+v"(x3) : "v"(a), "s"(sb) : "s20", "s21"); \
    asm volatile(INSTR : "+v"(x4) : "v"(a), "s"(sb) : "s20", "s21"); asm volatile(INSTR : "+v"(x5) : "v"(a), "s"(sb) : "s20", "s21"); \
    asm volatile(INSTR : "+v"(x6) : "v"(a), "s"(sb) : "s20", "s21"); asm volatile(INSTR : "+v"(x7) : "v"(a), "s"(sb) : "s20", "s21");

__global__ void p_pair_test_mix(float *out, unsigned long long *clocks, float a, float sb, int iters)
{
    unsigned long long c0 = 0, w0 = 0;
    const bool sampler = clocks != nullptr && blockIdx.x == 0 && threadIdx.x == 0;
    if (sampler) { c0 = clock64(); w0 = wall_clock64(); }
    float x0 = threadIdx.x, x1 = x0 + 1, x2 = x0 + 2, x3 = x0 + 3, x4 = x0 + 4, x5 = x0 + 5, x6 = x0 + 6, x7 = x0 + 7;
    for (int i = 0; i < iters; ++i) {
        ON_ALL_CHAINS("v_min_f32 %0, %2, %0")
        ON_ALL_CHAINS("v_max_f32 %0, %2, %0")
        ON_ALL_CHAINS("v_sub_f32 %0, %1, %0")
        ON_ALL_CHAINS("v_add_f32 %0, 1.0, %0")
        ON_ALL_CHAINS("v_min_f32 %0, %2, %0")
        ON_ALL_CHAINS("v_max_f32 %0, %2, %0")
        ON_ALL_CHAINS("v_sub_f32 %0, %1, %0")
        ON_ALL_CHAINS("v_add_f32_e64 %0, %1, %0 clamp")
        ON_ALL_CHAINS("v_mul_f32 %0, %1, %0")
        ON_ALL_CHAINS("v_cmp_ge_f32 s[20:21], %1, %0")
    }
    out[blockIdx.x * blockDim.x + threadIdx.x] = x0 + x1 + x2 + x3 + x4 + x5 + x6 + x7;
    if (sampler) {
        clocks[0] = clock64() - c0;
        clocks[1] = wall_clock64() - w0;
    }
}

typedef void (*probe_fn)(float *, unsigned long long *, float, float, int);

struct Probe {
    const char *name;
    probe_fn fn;
    int per_trip = 64;  // instructions per lane and loop trip
};

// the first seven are the pair test's own instructions, the eighth their mix (bench.py's default calibration)
const Probe kProbes[] = {
    {"v_sub_f32 v,v", p_sub_vv},
    {"v_add_f32 1.0,v", p_add_const},
    {"v_add_f32 v,v clamp", p_add_clamp},
    {"v_mul_f32 v,v", p_mul_vv},
    {"v_min_f32 s,v", p_min_sv},
    {"v_max_f32 s,v", p_max_sv},
    {"v_cmp_ge_f32 sgpr-pair", p_cmp_sgpr},
    {"pair-test mix (10 instructions)", p_pair_test_mix, 80},
    {"v_add_f32 v,v", p_add_vv},
    {"v_add_f32 s,v", p_add_sv},
    {"v_min_f32 v,v", p_min_vv},
    {"v_max_f32 v,v", p_max_vv},
    {"v_cmp_ge_f32 vcc", p_cmp_vcc},
    {"v_mov_b32", p_mov},
    {"v_fma_f32 a,x,x", p_fma},
    {"v_fma_f32 x,a,1.0", p_fma_const},
    {"v_fmac_f32", p_fmac},
    {"v_max3_f32", p_max3},
    {"v_min_i32", p_min_i32},
    {"v_max_u32", p_max_u32},
    {"v_and_b32", p_and},
    {"v_add_u32", p_add_u32},
    {"v_mul_f32 |abs|", p_mul_abs},
    {"v_sub_f32 clamp", p_sub_clamp},
    {"v_mul_f32 clamp", p_mul_clamp},
    {"v_rcp_f32", p_rcp},
    {"v_mul_f64", p_mul_f64},
    {"v_fma_f64", p_fma_f64},
    {"v_cmp_ge_f64", p_cmp_f64},
    {"v_cvt_f64_f32", p_cvt_f64_f32},
    {"v_cmp_lt_u64", p_cmp_lt_u64},
    {"v_cmp_lt_u32", p_cmp_lt_u32},
    {"v_readlane_b32", p_readlane},
};
constexpr int kProbeCount = (int)(sizeof(kProbes) / sizeof(kProbes[0]));

}  // namespace

extern "C" {

int valu_probe_count(void) { return kProbeCount; }

const char *valu_probe_name(int i) { return (i >= 0 && i < kProbeCount) ? kProbes[i].name : ""; }

// Lane-instructions of the probed kind that one launch of probe i executes.
double valu_probe_lane_ops(int i, int blocks, int iters)
{
    if (i < 0 || i >= kProbeCount) return 0.0;
    return (double)blocks * 256.0 * (double)iters * (double)kProbes[i].per_trip;
}

// Enqueues probe i on `stream`: `blocks` workgroups of 256 threads.  out: device, blocks * 256 floats.
// clocks: device, two 64-bit words (shader-clock ticks and wall-clock ticks of one wavefront), or NULL.
// Returns the hipError_t of the launch as an int (0 = ok), -1 for a bad argument.
int valu_probe_run(int i, int blocks, int iters, float *out, unsigned long long *clocks, void *stream)
{
    if (i < 0 || i >= kProbeCount || blocks <= 0 || blocks > 65535 || iters < 0 || iters > 1000000 || !out) return -1;
    (void)hipGetLastError();
    kProbes[i].fn<<<dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream)>>>(out, clocks, 1.5f, 0.25f, iters);
    return (int)hipGetLastError();
}

}  // extern "C"
