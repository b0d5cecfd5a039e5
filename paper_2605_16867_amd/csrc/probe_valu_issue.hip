// Measuring aid, not part of libgoodroute: how fast one SIMD of a gfx950 compute unit issues
// vector-ALU instructions of different kinds, alone and in the mix of the scoring kernel's main
// pass (two multiply-adds and one three-way minimum per two pairs).  The figures back the issue
// model that the scoring kernel's roofline is read against.
//
//   hipcc --offload-arch=gfx950 -O3 -o probe_valu_issue probe_valu_issue.hip && ./probe_valu_issue
//
// Every case runs the same way: 256 compute units x 4 SIMDs x 6 waves, each wave a loop of 64
// copies of the instruction (or 32 copies of the triple) on eight independent accumulators, so
// that neither dependencies nor occupancy limit the rate.  Reported: wave instructions per second
// per SIMD and the shader cycles each takes, with the shader clock read back from the hardware
// counter over the same run.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

#define CHECK(x)                                                                      \
    do {                                                                              \
        hipError_t e_ = (x);                                                          \
        if (e_ != hipSuccess) { printf("%s: %s\n", #x, hipGetErrorString(e_)); exit(1); } \
    } while (0)

// 64 copies of one instruction in a single asm block (the compiler puts nothing in between):
// I(acc) gives the instruction's text for accumulator operand `acc`; %8 %9 are vector inputs,
// %10 a scalar input, %11 a lane mask in a scalar pair.
#define ROUND(I) I("%0") I("%1") I("%2") I("%3") I("%4") I("%5") I("%6") I("%7")
#define BODY64(I)                                                                                          \
    asm volatile(ROUND(I) ROUND(I) ROUND(I) ROUND(I) ROUND(I) ROUND(I) ROUND(I) ROUND(I)                    \
                 : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(a[4]), "+v"(a[5]), "+v"(a[6]), "+v"(a[7]) \
                 : "v"(x), "v"(y), "s"(sc), "s"(mask)                                                       \
                 : "vcc", "s20")

#define I_FMA_V(r) "v_fma_f32 " r ", %8, %9, " r "\n"
#define I_FMA_S(r) "v_fma_f32 " r ", %10, %9, " r "\n"
#define I_FMAC(r) "v_fmac_f32 " r ", %8, %9\n"
#define I_ADD(r) "v_add_f32 " r ", %8, " r "\n"
#define I_MUL(r) "v_mul_f32 " r ", %8, " r "\n"
#define I_AND(r) "v_and_b32 " r ", %8, " r "\n"
#define I_ADDU(r) "v_add_u32 " r ", %8, " r "\n"
#define I_MOV(r) "v_mov_b32 " r ", %8\n"
#define I_MIN3(r) "v_min3_f32 " r ", " r ", %8, %9\n"
#define I_MIN(r) "v_min_f32 " r ", %8, " r "\n"
#define I_MED3U(r) "v_med3_u32 " r ", " r ", %8, %9\n"
#define I_MINU(r) "v_min_u32 " r ", %8, " r "\n"
#define I_LSHLADD(r) "v_lshl_add_u32 " r ", " r ", 1, %8\n"
#define I_CVT(r) "v_cvt_f32_i32 " r ", %8\n"
#define I_CMP(r) "v_cmp_lt_f32 vcc, %8, " r "\n"
#define I_CND32(r) "v_cndmask_b32_e32 " r ", %8, %9, vcc\n"
#define I_CND64(r) "v_cndmask_b32_e64 " r ", %8, %9, %11\n"
#define I_DPPMOV(r) "v_mov_b32_dpp " r ", %8 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n"
#define I_DPPMIN(r) "v_min_f32_dpp " r ", %8, " r " row_shr:1 row_mask:0xf bank_mask:0xf\n"
#define I_READLANE(r) "v_readlane_b32 s20, %8, 3\n"
// the main pass's triple: two multiply-adds into temporaries (%12 %13), one three-way minimum
#define I_TRIPLE_V(r) "v_fma_f32 %12, %8, %9, %14\n v_fma_f32 %13, %8, %14, %9\n v_min3_f32 " r ", " r ", %12, %13\n"
#define I_TRIPLE_S(r) "v_fma_f32 %12, %10, %9, %14\n v_fma_f32 %13, %10, %14, %9\n v_min3_f32 " r ", " r ", %12, %13\n"
#define BODY_TRIPLES(I)                                                                                    \
    asm volatile(ROUND(I) ROUND(I) ROUND(I) ROUND(I)                                                        \
                 : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(a[4]), "+v"(a[5]), "+v"(a[6]), "+v"(a[7]) \
                 : "v"(x), "v"(y), "s"(sc), "s"(mask), "v"(t0v), "v"(t1v), "v"(z))
#define I_FMA64(r) "v_fma_f64 " r ", %8, %8, " r "\n"

constexpr int kIters = 20000;
constexpr int kPerIter = 64;

template <int kCase>
__global__ __launch_bounds__(384) __attribute__((amdgpu_waves_per_eu(6, 6))) void k(float* out, const float* in)
{
    float x = in[threadIdx.x], y = in[threadIdx.x + 64], z = in[threadIdx.x + 192];
    float sc = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(in[700])));
    unsigned long long mask = __ballot(in[threadIdx.x] > 0.5f);
    float a[8], t0v = 0.f, t1v = 0.f;
    double d[8];
    const double dx = (double)x;
#pragma unroll
    for (int j = 0; j < 8; ++j) { a[j] = in[128 + j]; d[j] = (double)in[136 + j]; }
    for (int i = 0; i < kIters; ++i) {
        if (kCase == 0) BODY64(I_FMA_V);
        if (kCase == 1) BODY64(I_FMA_S);
        if (kCase == 2) BODY64(I_FMAC);
        if (kCase == 3) BODY64(I_ADD);
        if (kCase == 4) BODY64(I_MUL);
        if (kCase == 5) BODY64(I_AND);
        if (kCase == 6) BODY64(I_ADDU);
        if (kCase == 7) BODY64(I_MOV);
        if (kCase == 8) BODY64(I_MIN3);
        if (kCase == 9) BODY64(I_MIN);
        if (kCase == 10) BODY64(I_MED3U);
        if (kCase == 11) BODY64(I_MINU);
        if (kCase == 12) BODY64(I_LSHLADD);
        if (kCase == 13) BODY64(I_CVT);
        if (kCase == 14) BODY64(I_CMP);
        if (kCase == 15) BODY64(I_CND32);
        if (kCase == 16) BODY64(I_CND64);
        if (kCase == 17) BODY64(I_DPPMOV);
        if (kCase == 18) BODY64(I_DPPMIN);
        if (kCase == 19) BODY64(I_READLANE);
        if (kCase == 20)
            asm volatile(ROUND(I_FMA64) ROUND(I_FMA64) ROUND(I_FMA64) ROUND(I_FMA64) ROUND(I_FMA64) ROUND(I_FMA64)
                             ROUND(I_FMA64) ROUND(I_FMA64)
                         : "+v"(d[0]), "+v"(d[1]), "+v"(d[2]), "+v"(d[3]), "+v"(d[4]), "+v"(d[5]), "+v"(d[6]), "+v"(d[7])
                         : "v"(dx));
        if (kCase == 21) BODY_TRIPLES(I_TRIPLE_V);
        if (kCase == 22) BODY_TRIPLES(I_TRIPLE_S);
    }
    float s = t0v + t1v;
#pragma unroll
    for (int j = 0; j < 8; ++j) s += a[j] + (float)d[j];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

struct Case {
    const char* name;
    void (*kernel)(float*, const float*);
    int per_iter;
};

int main()
{
    const Case cases[] = {
        {"v_fma_f32 (vector operands)", k<0>, kPerIter}, {"v_fma_f32 (one scalar operand)", k<1>, kPerIter},
        {"v_fmac_f32", k<2>, kPerIter}, {"v_add_f32", k<3>, kPerIter}, {"v_mul_f32", k<4>, kPerIter},
        {"v_and_b32", k<5>, kPerIter}, {"v_add_u32", k<6>, kPerIter}, {"v_mov_b32", k<7>, kPerIter},
        {"v_min3_f32", k<8>, kPerIter}, {"v_min_f32", k<9>, kPerIter}, {"v_med3_u32", k<10>, kPerIter},
        {"v_min_u32", k<11>, kPerIter}, {"v_lshl_add_u32", k<12>, kPerIter}, {"v_cvt_f32_i32", k<13>, kPerIter},
        {"v_cmp_lt_f32 -> vcc", k<14>, kPerIter}, {"v_cndmask_b32 e32 (mask in vcc)", k<15>, kPerIter},
        {"v_cndmask_b32 e64 (mask in a scalar pair)", k<16>, kPerIter}, {"v_mov_b32_dpp quad_perm", k<17>, kPerIter},
        {"v_min_f32_dpp row_shr:1", k<18>, kPerIter}, {"v_readlane_b32", k<19>, kPerIter},
        {"v_fma_f64", k<20>, kPerIter},
        {"triple fma, fma, min3 (vector operands)", k<21>, 96}, {"triple fma, fma, min3 (scalar operand)", k<22>, 96},
    };
    hipDeviceProp_t prop;
    CHECK(hipGetDeviceProperties(&prop, 0));
    const int cus = prop.multiProcessorCount, blocks = cus * 4;        // 4 workgroups of 6 waves per compute unit
    float *in, *out;
    CHECK(hipMalloc(&in, 1024 * sizeof(float)));
    CHECK(hipMalloc(&out, (size_t)blocks * 384 * sizeof(float)));
    float host[1024];
    for (int i = 0; i < 1024; ++i) host[i] = 1.0f + (float)(i % 7) * 0.125f;
    CHECK(hipMemcpy(in, host, sizeof(host), hipMemcpyHostToDevice));
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    printf("%d compute units, %d workgroups of 6 waves, %d iterations\n", cus, blocks, kIters);
    // Two passes over the cases; the first only brings the clocks up.  One issue slot = the time a
    // single-issue instruction (v_min3_f32) takes in the second pass: four shader cycles.
    constexpr int kCases = sizeof(cases) / sizeof(cases[0]);
    double rate[kCases];
    for (int pass = 0; pass < 2; ++pass) {
        for (int c = 0; c < kCases; ++c) {
            hipLaunchKernelGGL(cases[c].kernel, dim3(blocks), dim3(384), 0, 0, out, in);     // warm-up
            CHECK(hipEventRecord(e0, 0));
            hipLaunchKernelGGL(cases[c].kernel, dim3(blocks), dim3(384), 0, 0, out, in);
            CHECK(hipEventRecord(e1, 0));
            CHECK(hipEventSynchronize(e1));
            float ms = 0.f;
            CHECK(hipEventElapsedTime(&ms, e0, e1));
            rate[c] = (double)kIters * cases[c].per_iter * 6.0 / (ms * 1e-3);     // wave instructions / s / SIMD
        }
    }
    const double slot_s = 1.0 / rate[8];
    printf("one issue slot (v_min3_f32 alone) = %.3f ns: four cycles at %.2f GHz\n", slot_s * 1e9, 4.0 / slot_s / 1e9);
    for (int c = 0; c < kCases; ++c)
        printf("%-44s %.3e wave-instr/s per SIMD = %5.2f issue slots = %5.2f cycles each\n", cases[c].name, rate[c],
               1.0 / rate[c] / slot_s, 4.0 / rate[c] / slot_s);
    return 0;
}
