// Issue cost of the vector instructions the iterated kernel is made of, on gfx950.
//
// Each case runs a long unrolled stream of one instruction pattern (registers named explicitly,
// values irrelevant, nothing loaded or stored inside the loop) with W waves per SIMD and prints
// the cycles one wave64 instruction costs the SIMD, assuming the 2.4 GHz engine clock.  The
// figures bound the arithmetic roofline of k_iter: see the per-step sum printed at the end.
//
// Build: hipcc --offload-arch=gfx950 -O3 valu_probe.hip -o valu_probe     Run: ./valu_probe
#include <hip/hip_runtime.h>

#include <cstdio>

#define CHECK(x)                                                       \
    do {                                                               \
        if ((x) != hipSuccess) {                                       \
            std::printf("HIP error at line %d\n", __LINE__);           \
            return 1;                                                  \
        }                                                              \
    } while (0)

namespace {

constexpr int kIters = 2048;
constexpr double kClockHz = 2.4e9;

#define REP4(X) X X X X
#define REP8(X) X X X X X X X X
#define CLOB                                                                                                  \
    "v100", "v101", "v102", "v103", "v104", "v105", "v106", "v107", "v108", "v109", "v110", "v111", "v112",   \
        "v113", "v114", "v115", "v116", "v117", "v118", "v119"
#define FMA4                                                                                     \
    "v_fma_f32 v100, v105, v106, v107\n v_fma_f32 v101, v104, v110, v111\n"                      \
    "v_fma_f32 v102, v108, v109, v115\n v_fma_f32 v103, v112, v113, v114\n"
#define FMA3 "v_fma_f32 v100, v105, v106, v107\n v_fma_f32 v101, v104, v110, v111\n v_fma_f32 v102, v108, v109, v115\n"

enum Case {
    kFma, kMul, kErrPair, kCvtTo, kCvtFrom, kRcp, kMin3, kCmpSel, kFmaWithCvtTo, kFmaWithCvtFrom, kFmaWithMin3, kCases
};

template <int OP>
__global__ __launch_bounds__(256) void k_stream(float *out)
{
    asm volatile(
        "v_mov_b32 v100, 0.5\n v_mov_b32 v101, 0.5\n v_mov_b32 v102, 0.5\n v_mov_b32 v103, 0.5\n v_mov_b32 v104, 0.5\n"
        "v_mov_b32 v105, 0.5\n v_mov_b32 v106, 0.5\n v_mov_b32 v107, 0.5\n v_mov_b32 v108, 0.5\n v_mov_b32 v109, 0.5\n"
        "v_mov_b32 v110, 0.5\n v_mov_b32 v111, 0.5\n v_mov_b32 v112, 0.5\n v_mov_b32 v113, 0.5\n v_mov_b32 v114, 0.5\n"
        "v_mov_b32 v115, 0.5\n v_mov_b32 v116, 0.5\n v_mov_b32 v117, 0.5\n v_mov_b32 v118, 0.5\n v_mov_b32 v119, 0.5\n" ::
            : CLOB);
    for (int it = 0; it < kIters; ++it) {      // every case: 32 instructions per trip
        if constexpr (OP == kFma) asm volatile(REP8(FMA4)::: CLOB);
        if constexpr (OP == kMul)
            asm volatile(REP8("v_mul_f32 v100, v105, v106\n v_mul_f32 v101, v104, v110\n v_mul_f32 v102, v108, v109\n"
                              "v_mul_f32 v103, v112, v113\n")::
                             : CLOB);
        if constexpr (OP == kErrPair)          // residual, then square-accumulate, for two stored-scale candidates
            asm volatile(REP8("v_fma_f32 v108, v105, v116, v106\n v_fmac_f32 v100, v108, v108\n"
                              "v_fma_f32 v109, v105, v112, v106\n v_fmac_f32 v101, v109, v109\n")::
                             : CLOB);
        if constexpr (OP == kCvtTo)
            asm volatile(REP8("v_cvt_scalef32_pk_fp4_f32 v100, v105, v106, 1.0\n v_cvt_scalef32_pk_fp4_f32 v101, v105, v106, 1.0\n"
                              "v_cvt_scalef32_pk_fp4_f32 v102, v105, v106, 1.0\n v_cvt_scalef32_pk_fp4_f32 v103, v105, v106, 1.0\n")::
                             : CLOB);
        if constexpr (OP == kCvtFrom)
            asm volatile(REP8("v_cvt_scalef32_pk_f32_fp4 v[100:101], v105, 1.0\n v_cvt_scalef32_pk_f32_fp4 v[102:103], v106, 1.0\n"
                              "v_cvt_scalef32_pk_f32_fp4 v[108:109], v107, 1.0\n v_cvt_scalef32_pk_f32_fp4 v[110:111], v104, 1.0\n")::
                             : CLOB);
        if constexpr (OP == kRcp)
            asm volatile(REP8("v_rcp_f32 v100, v105\n v_rcp_f32 v101, v105\n v_rcp_f32 v102, v105\n v_rcp_f32 v103, v105\n")::: CLOB);
        if constexpr (OP == kMin3)
            asm volatile(REP8("v_min3_f32 v100, v100, v105, v101\n v_min3_f32 v101, v101, v105, v102\n"
                              "v_min3_f32 v102, v102, v105, v103\n v_min3_f32 v103, v103, v105, v100\n")::
                             : CLOB);
        if constexpr (OP == kCmpSel)
            asm volatile(REP8("v_cmp_lt_f32 vcc, v100, v101\n v_cndmask_b32 v102, v102, v103, vcc\n"
                              "v_cmp_lt_f32 vcc, v101, v100\n v_cndmask_b32 v103, v103, v102, vcc\n")::
                             : "vcc", CLOB);
        if constexpr (OP == kFmaWithCvtTo)
            asm volatile(REP4(FMA4 FMA3 "v_cvt_scalef32_pk_fp4_f32 v116, v117, v118, 1.0\n")::: CLOB);
        if constexpr (OP == kFmaWithCvtFrom)
            asm volatile(REP4(FMA4 FMA3 "v_cvt_scalef32_pk_f32_fp4 v[116:117], v118, 1.0\n")::: CLOB);
        if constexpr (OP == kFmaWithMin3) asm volatile(REP4(FMA4 FMA3 "v_min3_f32 v116, v117, v118, v119\n")::: CLOB);
    }
    float r;
    asm volatile("v_add_f32 %0, v100, v101\n v_add_f32 %0, %0, v102\n v_add_f32 %0, %0, v103\n v_add_f32 %0, %0, v116"
                 : "=v"(r)
                 :
                 : CLOB);
    out[blockIdx.x * 256 + threadIdx.x] = r;
}

template <int OP>
int run(float *out, int waves_per_simd, double *cycles)
{
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    const int grid = 256 * waves_per_simd;      // one 4-wave workgroup per compute unit and wave slot
    hipLaunchKernelGGL(k_stream<OP>, dim3(grid), dim3(256), 0, 0, out);
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(e0, 0));
    hipLaunchKernelGGL(k_stream<OP>, dim3(grid), dim3(256), 0, 0, out);
    CHECK(hipEventRecord(e1, 0));
    CHECK(hipDeviceSynchronize());
    float ms = 0.0f;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    *cycles = ms * 1e-3 * kClockHz / ((double)waves_per_simd * kIters * 32);
    CHECK(hipEventDestroy(e0));
    CHECK(hipEventDestroy(e1));
    return 0;
}

}  // namespace

int main()
{
    float *out = nullptr;
    CHECK(hipMalloc(&out, sizeof(float) * 256 * 8 * 256));
    const char *names[kCases] = {"v_fma_f32, independent",
                                 "v_mul_f32",
                                 "error pair (v_fma_f32 + v_fmac_f32)",
                                 "v_cvt_scalef32_pk_fp4_f32",
                                 "v_cvt_scalef32_pk_f32_fp4",
                                 "v_rcp_f32",
                                 "v_min3_f32",
                                 "v_cmp_lt_f32 + v_cndmask_b32",
                                 "7 v_fma_f32 + 1 cvt to fp4",
                                 "7 v_fma_f32 + 1 cvt from fp4",
                                 "7 v_fma_f32 + 1 v_min3_f32"};
    for (int w : {6, 2, 1}) {
        double c[kCases];
        if (run<kFma>(out, w, &c[kFma]) || run<kMul>(out, w, &c[kMul]) || run<kErrPair>(out, w, &c[kErrPair]) ||
            run<kCvtTo>(out, w, &c[kCvtTo]) || run<kCvtFrom>(out, w, &c[kCvtFrom]) || run<kRcp>(out, w, &c[kRcp]) ||
            run<kMin3>(out, w, &c[kMin3]) || run<kCmpSel>(out, w, &c[kCmpSel]) ||
            run<kFmaWithCvtTo>(out, w, &c[kFmaWithCvtTo]) || run<kFmaWithCvtFrom>(out, w, &c[kFmaWithCvtFrom]) ||
            run<kFmaWithMin3>(out, w, &c[kFmaWithMin3]))
            return 1;
        std::printf("waves per SIMD: %d\n", w);
        for (int k = 0; k < kCases; ++k) std::printf("  %-40s %.2f cycles per wave64 instruction\n", names[k], c[k]);
        if (w == 6) {
            // one beta step of the bracket search: 2 + 16 products, 8 + 8 conversions, 1 estimate + 2 Newton
            // operations, 2 x 16 error pairs, minimum / compare / select
            const double alone = 18 * c[kMul] + 8 * c[kCvtTo] + 8 * c[kCvtFrom] + c[kRcp] + 2 * c[kFma] +
                                 32 * 2 * c[kErrPair] + c[kMin3] + 2 * c[kCmpSel];
            const double single = 18 * 4 + 8 * c[kCvtTo] + 8 * c[kCvtFrom] + c[kRcp] + 2 * 4 + 64 * 4 + 3 * 4;
            std::printf("  one beta step, every instruction at its stand-alone cost: %.0f cycles\n", alone);
            std::printf("  one beta step, plain arithmetic at 4 cycles (no pairing of two waves): %.0f cycles\n", single);
        }
        std::fflush(stdout);
    }
    CHECK(hipFree(out));
    return 0;
}
