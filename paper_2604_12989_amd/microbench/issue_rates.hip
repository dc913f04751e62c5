// Issue-rate measurements behind the attention kernel's design (gfx950): cycles per instruction of
// the vector operations a softmax needs, what a wave can issue beside its own matrix instructions,
// and how two waves of one SIMD share it.  Not part of the library; build and run by hand:
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 -Xclang -target-feature -Xclang -packed-fp32-ops \
//       paper_2604_12989_amd/microbench/issue_rates.hip -o /tmp/issue_rates && /tmp/issue_rates
// One workgroup of eight waves (waves w and w + 4 share SIMD w); every wave runs `iters` iterations
// of a fixed instruction block between two reads of the cycle counter.  "wave0" is the older wave
// of its SIMD (it wins the issue arbitration), "wave4" the younger: when both run the same block,
// wave4's time is when the SIMD has finished both.  grid 256 repeats the measurement with every
// compute unit busy (the clock then drops: see the MHz column).
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdint>
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

#define REP4(x) x x x x
#define REP8(x) REP4(x) REP4(x)
#define REP16(x) REP8(x) REP8(x)
#define REP32(x) REP16(x) REP16(x)

__device__ __forceinline__ uint64_t memtime()
{
    uint64_t t;
    asm volatile("s_memtime %0\n\ts_waitcnt lgkmcnt(0)" : "=s"(t)::"memory");
    return t;
}
__device__ __forceinline__ uint64_t realtime()
{
    uint64_t t;
    asm volatile("s_memrealtime %0\n\ts_waitcnt lgkmcnt(0)" : "=s"(t)::"memory");
    return t;
}

// MODE: what group 0 (waves 0-3) runs / what group 1 (waves 4-7) runs, encoded in the body below.
template <int MODE>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void k(uint64_t *out, int iters, float seed)
{
    const int wave = threadIdx.x >> 6;
    const int grp = wave >> 2;
    float x0 = seed + threadIdx.x * 1e-3f, x1 = x0 + 1.f, x2 = x0 + 2.f, x3 = x0 + 3.f;
    float y0 = 0, y1 = 0, y2 = 0, y3 = 0, y4 = 0, y5 = 0, y6 = 0, y7 = 0;
    unsigned p0 = 0, p1 = 0, p2 = 0, p3 = 0;
    floatx16 a0, a1, a2, a3;
    for (int v = 0; v < 16; ++v) a0[v] = a1[v] = a2[v] = a3[v] = 0.f;
    bf16x8 ka, kb;
    for (int j = 0; j < 8; ++j) { ka[j] = (__bf16)(float)(threadIdx.x + j); kb[j] = (__bf16)1.0f; }
    __syncthreads();
    const uint64_t t0 = memtime(), r0 = realtime();
#define EXP4 "v_exp_f32 %0, %8\n\tv_exp_f32 %1, %9\n\tv_exp_f32 %2, %10\n\tv_exp_f32 %3, %11\n\t"
#define EXP4b "v_exp_f32 %4, %8\n\tv_exp_f32 %5, %9\n\tv_exp_f32 %6, %10\n\tv_exp_f32 %7, %11\n\t"
#define FMA4 "v_fma_f32 %0, %8, %9, %10\n\tv_fma_f32 %1, %9, %10, %11\n\tv_fma_f32 %2, %10, %11, %8\n\tv_fma_f32 %3, %11, %8, %9\n\t"
#define FMA4b "v_fma_f32 %4, %8, %9, %10\n\tv_fma_f32 %5, %9, %10, %11\n\tv_fma_f32 %6, %10, %11, %8\n\tv_fma_f32 %7, %11, %8, %9\n\t"
#define MAX4 "v_max3_f32 %0, %8, %9, %10\n\tv_max3_f32 %1, %9, %10, %11\n\tv_max3_f32 %2, %10, %11, %8\n\tv_max3_f32 %3, %11, %8, %9\n\t"
#define CVT4 "v_cvt_pk_bf16_f32 %0, %8, %9\n\tv_cvt_pk_bf16_f32 %1, %9, %10\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %3, %11, %8\n\t"
#define DOT4 "v_dot2c_f32_bf16 %0, %8, %9\n\tv_dot2c_f32_bf16 %1, %9, %10\n\tv_dot2c_f32_bf16 %2, %10, %11\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"
#define VOPS(body) asm volatile(body : "+v"(y0), "+v"(y1), "+v"(y2), "+v"(y3), "+v"(y4), "+v"(y5), "+v"(y6), "+v"(y7) : "v"(x0), "v"(x1), "v"(x2), "v"(x3))
#define MF(acc) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, kb, acc, 0, 0, 0)
    // every mode: `iters` iterations of a block; per block the count of "units" is fixed below
    for (int it = 0; it < iters; ++it) {
        if (MODE == 0) { VOPS(REP4(EXP4 EXP4b)); }                        // 32 exp
        if (MODE == 1) { VOPS(REP4(FMA4 FMA4b)); }                        // 32 fma
        if (MODE == 2) { VOPS(REP8(MAX4)); }                              // 32 max3
        if (MODE == 3) { VOPS(REP8(CVT4)); }                              // 32 cvt_pk
        if (MODE == 4) { VOPS(REP8(DOT4)); }                              // 32 dot2c
        if (MODE == 5) {                                                  // 8 mfma, 4 accumulators
            MF(a0); MF(a1); MF(a2); MF(a3); MF(a0); MF(a1); MF(a2); MF(a3);
        }
        if (MODE == 6) {                                                  // 8 x (mfma + 4 fma)
#define U6(acc) MF(acc); VOPS(FMA4); __builtin_amdgcn_sched_barrier(0);
            U6(a0) U6(a1) U6(a2) U6(a3) U6(a0) U6(a1) U6(a2) U6(a3)
        }
        if (MODE == 7) {                                                  // 8 x (mfma + 6 fma)
#define U7(acc) MF(acc); VOPS(FMA4 "v_fma_f32 %4, %8, %9, %10\n\tv_fma_f32 %5, %9, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0);
            U7(a0) U7(a1) U7(a2) U7(a3) U7(a0) U7(a1) U7(a2) U7(a3)
        }
        if (MODE == 8) {                                                  // 8 x (mfma + 8 fma)
#define U8(acc) MF(acc); VOPS(FMA4 FMA4b); __builtin_amdgcn_sched_barrier(0);
            U8(a0) U8(a1) U8(a2) U8(a3) U8(a0) U8(a1) U8(a2) U8(a3)
        }
        if (MODE == 9) {                                                  // 8 x (mfma + 1 exp)
#define U9(acc) MF(acc); VOPS("v_exp_f32 %0, %8\n\t"); __builtin_amdgcn_sched_barrier(0);
            U9(a0) U9(a1) U9(a2) U9(a3) U9(a0) U9(a1) U9(a2) U9(a3)
        }
        if (MODE == 10) {                                                 // 8 x (mfma + 2 exp)
#define U10(acc) MF(acc); VOPS("v_exp_f32 %0, %8\n\tv_exp_f32 %1, %9\n\t"); __builtin_amdgcn_sched_barrier(0);
            U10(a0) U10(a1) U10(a2) U10(a3) U10(a0) U10(a1) U10(a2) U10(a3)
        }
        if (MODE == 11) {                                                 // 8 x (mfma + 1 exp + 2 fma + half cvt, dot): lean softmax mix
#define U11(acc) MF(acc); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0);
            U11(a0) U11(a1) U11(a2) U11(a3) U11(a0) U11(a1) U11(a2) U11(a3)
        }
        if (MODE == 12) {                                                 // group 0: mfma only; group 1: fma only
            if (grp == 0) { MF(a0); MF(a1); MF(a2); MF(a3); MF(a0); MF(a1); MF(a2); MF(a3); }
            else { VOPS(REP4(FMA4 FMA4b)); }
        }
        if (MODE == 13) {                                                 // group 0: mfma only; group 1: exp only
            if (grp == 0) { MF(a0); MF(a1); MF(a2); MF(a3); MF(a0); MF(a1); MF(a2); MF(a3); }
            else { VOPS(REP4(EXP4 EXP4b)); }
        }
        if (MODE == 14) {                                                 // group 0: mfma only; group 1: the lean mix without mfma
            if (grp == 0) { MF(a0); MF(a1); MF(a2); MF(a3); MF(a0); MF(a1); MF(a2); MF(a3); }
            else { VOPS(REP8("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t")); }
        }
        if (MODE == 15) {                                                 // both groups: 16 mfma then softmax-like 16 x (fma, exp) + 8 cvt + 8 dot
            MF(a0); MF(a1); MF(a2); MF(a3); MF(a0); MF(a1); MF(a2); MF(a3);
            MF(a0); MF(a1); MF(a2); MF(a3); MF(a0); MF(a1); MF(a2); MF(a3);
            VOPS(REP4(FMA4 EXP4b) REP8("v_cvt_pk_bf16_f32 %2, %10, %11\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"));
        }
        if (MODE == 16) {                                                 // same totals, group 1 runs the two halves in the other order
            if (grp == 1) VOPS(REP4(FMA4 EXP4b) REP8("v_cvt_pk_bf16_f32 %2, %10, %11\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"));
            MF(a0); MF(a1); MF(a2); MF(a3); MF(a0); MF(a1); MF(a2); MF(a3);
            MF(a0); MF(a1); MF(a2); MF(a3); MF(a0); MF(a1); MF(a2); MF(a3);
            if (grp == 0) VOPS(REP4(FMA4 EXP4b) REP8("v_cvt_pk_bf16_f32 %2, %10, %11\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"));
        }
        if (MODE == 17) {                                                 // both groups: 16 x (mfma + lean mix), fine interleave
            U11(a0) U11(a1) U11(a2) U11(a3) U11(a0) U11(a1) U11(a2) U11(a3)
            U11(a0) U11(a1) U11(a2) U11(a3) U11(a0) U11(a1) U11(a2) U11(a3)
        }
        if (MODE == 20) { MF(a0); VOPS("v_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a0); VOPS("v_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); }
        if (MODE == 21) { MF(a0); VOPS("v_dot2c_f32_bf16 %3, %11, %8\n\tv_dot2c_f32_bf16 %3, %11, %8\n\tv_dot2c_f32_bf16 %3, %11, %8\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_dot2c_f32_bf16 %3, %11, %8\n\tv_dot2c_f32_bf16 %3, %11, %8\n\tv_dot2c_f32_bf16 %3, %11, %8\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_dot2c_f32_bf16 %3, %11, %8\n\tv_dot2c_f32_bf16 %3, %11, %8\n\tv_dot2c_f32_bf16 %3, %11, %8\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_dot2c_f32_bf16 %3, %11, %8\n\tv_dot2c_f32_bf16 %3, %11, %8\n\tv_dot2c_f32_bf16 %3, %11, %8\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a0); VOPS("v_dot2c_f32_bf16 %3, %11, %8\n\tv_dot2c_f32_bf16 %3, %11, %8\n\tv_dot2c_f32_bf16 %3, %11, %8\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_dot2c_f32_bf16 %3, %11, %8\n\tv_dot2c_f32_bf16 %3, %11, %8\n\tv_dot2c_f32_bf16 %3, %11, %8\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_dot2c_f32_bf16 %3, %11, %8\n\tv_dot2c_f32_bf16 %3, %11, %8\n\tv_dot2c_f32_bf16 %3, %11, %8\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_dot2c_f32_bf16 %3, %11, %8\n\tv_dot2c_f32_bf16 %3, %11, %8\n\tv_dot2c_f32_bf16 %3, %11, %8\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); }
        if (MODE == 22) { MF(a0); VOPS("v_max3_f32 %7, %8, %9, %10\n\tv_max3_f32 %7, %8, %9, %10\n\tv_max3_f32 %7, %8, %9, %10\n\tv_max3_f32 %7, %8, %9, %10\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_max3_f32 %7, %8, %9, %10\n\tv_max3_f32 %7, %8, %9, %10\n\tv_max3_f32 %7, %8, %9, %10\n\tv_max3_f32 %7, %8, %9, %10\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_max3_f32 %7, %8, %9, %10\n\tv_max3_f32 %7, %8, %9, %10\n\tv_max3_f32 %7, %8, %9, %10\n\tv_max3_f32 %7, %8, %9, %10\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_max3_f32 %7, %8, %9, %10\n\tv_max3_f32 %7, %8, %9, %10\n\tv_max3_f32 %7, %8, %9, %10\n\tv_max3_f32 %7, %8, %9, %10\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a0); VOPS("v_max3_f32 %7, %8, %9, %10\n\tv_max3_f32 %7, %8, %9, %10\n\tv_max3_f32 %7, %8, %9, %10\n\tv_max3_f32 %7, %8, %9, %10\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_max3_f32 %7, %8, %9, %10\n\tv_max3_f32 %7, %8, %9, %10\n\tv_max3_f32 %7, %8, %9, %10\n\tv_max3_f32 %7, %8, %9, %10\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_max3_f32 %7, %8, %9, %10\n\tv_max3_f32 %7, %8, %9, %10\n\tv_max3_f32 %7, %8, %9, %10\n\tv_max3_f32 %7, %8, %9, %10\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_max3_f32 %7, %8, %9, %10\n\tv_max3_f32 %7, %8, %9, %10\n\tv_max3_f32 %7, %8, %9, %10\n\tv_max3_f32 %7, %8, %9, %10\n\t"); __builtin_amdgcn_sched_barrier(0); }
        if (MODE == 23) { MF(a0); VOPS("v_exp_f32 %1, %9\n\tv_fma_f32 %0, %8, %9, %10\n\tv_fma_f32 %4, %9, %10, %11\n\tv_fma_f32 %5, %10, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_exp_f32 %1, %9\n\tv_fma_f32 %0, %8, %9, %10\n\tv_fma_f32 %4, %9, %10, %11\n\tv_fma_f32 %5, %10, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_exp_f32 %1, %9\n\tv_fma_f32 %0, %8, %9, %10\n\tv_fma_f32 %4, %9, %10, %11\n\tv_fma_f32 %5, %10, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_exp_f32 %1, %9\n\tv_fma_f32 %0, %8, %9, %10\n\tv_fma_f32 %4, %9, %10, %11\n\tv_fma_f32 %5, %10, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a0); VOPS("v_exp_f32 %1, %9\n\tv_fma_f32 %0, %8, %9, %10\n\tv_fma_f32 %4, %9, %10, %11\n\tv_fma_f32 %5, %10, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_exp_f32 %1, %9\n\tv_fma_f32 %0, %8, %9, %10\n\tv_fma_f32 %4, %9, %10, %11\n\tv_fma_f32 %5, %10, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_exp_f32 %1, %9\n\tv_fma_f32 %0, %8, %9, %10\n\tv_fma_f32 %4, %9, %10, %11\n\tv_fma_f32 %5, %10, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_exp_f32 %1, %9\n\tv_fma_f32 %0, %8, %9, %10\n\tv_fma_f32 %4, %9, %10, %11\n\tv_fma_f32 %5, %10, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); }
        if (MODE == 24) { MF(a0); VOPS("v_exp_f32 %1, %9\n\tv_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %6, %10\n\tv_fma_f32 %4, %9, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_exp_f32 %1, %9\n\tv_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %6, %10\n\tv_fma_f32 %4, %9, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_exp_f32 %1, %9\n\tv_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %6, %10\n\tv_fma_f32 %4, %9, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_exp_f32 %1, %9\n\tv_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %6, %10\n\tv_fma_f32 %4, %9, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a0); VOPS("v_exp_f32 %1, %9\n\tv_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %6, %10\n\tv_fma_f32 %4, %9, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_exp_f32 %1, %9\n\tv_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %6, %10\n\tv_fma_f32 %4, %9, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_exp_f32 %1, %9\n\tv_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %6, %10\n\tv_fma_f32 %4, %9, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_exp_f32 %1, %9\n\tv_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %6, %10\n\tv_fma_f32 %4, %9, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); }
        if (MODE == 25) { MF(a0); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_fma_f32 %4, %9, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_fma_f32 %4, %9, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_fma_f32 %4, %9, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_fma_f32 %4, %9, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a0); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_fma_f32 %4, %9, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_fma_f32 %4, %9, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_fma_f32 %4, %9, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_fma_f32 %4, %9, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); }
        if (MODE == 26) { MF(a0); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_fma_f32 %4, %9, %10, %11\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_fma_f32 %4, %9, %10, %11\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_fma_f32 %4, %9, %10, %11\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_fma_f32 %4, %9, %10, %11\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a0); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_fma_f32 %4, %9, %10, %11\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_fma_f32 %4, %9, %10, %11\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_fma_f32 %4, %9, %10, %11\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_fma_f32 %4, %9, %10, %11\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); }
        if (MODE == 27) { MF(a0); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_add_f32 %3, %3, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_add_f32 %3, %3, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_add_f32 %3, %3, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_add_f32 %3, %3, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a0); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_add_f32 %3, %3, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_add_f32 %3, %3, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_add_f32 %3, %3, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_add_f32 %3, %3, %11\n\t"); __builtin_amdgcn_sched_barrier(0); }
        if (MODE == 28) { MF(a0); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_add_f32 %3, %3, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_add_f32 %3, %3, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_add_f32 %3, %3, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_add_f32 %3, %3, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a0); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_add_f32 %3, %3, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_add_f32 %3, %3, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_add_f32 %3, %3, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_add_f32 %3, %3, %11\n\t"); __builtin_amdgcn_sched_barrier(0); }
        if (MODE == 29) { MF(a0); VOPS("v_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a0); VOPS("v_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); }
        if (MODE == 30) { MF(a0); VOPS("v_cvt_pk_bf16_f32 %2, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_cvt_pk_bf16_f32 %2, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_cvt_pk_bf16_f32 %2, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_cvt_pk_bf16_f32 %2, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a0); VOPS("v_cvt_pk_bf16_f32 %2, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_cvt_pk_bf16_f32 %2, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_cvt_pk_bf16_f32 %2, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_cvt_pk_bf16_f32 %2, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); }
        if (MODE == 31) { MF(a0); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_add_f32 %3, %3, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_fma_f32 %4, %9, %10, %11\n\tv_exp_f32 %6, %10\n\tv_add_f32 %7, %7, %10\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_add_f32 %3, %3, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_fma_f32 %4, %9, %10, %11\n\tv_exp_f32 %6, %10\n\tv_add_f32 %7, %7, %10\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a0); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_add_f32 %3, %3, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_fma_f32 %4, %9, %10, %11\n\tv_exp_f32 %6, %10\n\tv_add_f32 %7, %7, %10\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_add_f32 %3, %3, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_fma_f32 %4, %9, %10, %11\n\tv_exp_f32 %6, %10\n\tv_add_f32 %7, %7, %10\n\t"); __builtin_amdgcn_sched_barrier(0); }
        if (MODE == 32) { MF(a0); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_fma_f32 %4, %9, %10, %11\n\tv_exp_f32 %6, %10\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_fma_f32 %4, %9, %10, %11\n\tv_exp_f32 %6, %10\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a0); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_fma_f32 %4, %9, %10, %11\n\tv_exp_f32 %6, %10\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_fma_f32 %4, %9, %10, %11\n\tv_exp_f32 %6, %10\n\t"); __builtin_amdgcn_sched_barrier(0); }
        if (MODE == 33) { MF(a0); VOPS("v_dot2c_f32_bf16 %3, %11, %8\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_dot2c_f32_bf16 %3, %11, %8\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_dot2c_f32_bf16 %3, %11, %8\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_dot2c_f32_bf16 %3, %11, %8\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a0); VOPS("v_dot2c_f32_bf16 %3, %11, %8\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_dot2c_f32_bf16 %3, %11, %8\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_dot2c_f32_bf16 %3, %11, %8\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_dot2c_f32_bf16 %3, %11, %8\n\tv_dot2c_f32_bf16 %3, %11, %8\n\t"); __builtin_amdgcn_sched_barrier(0); }
        if (MODE == 34) { MF(a0); VOPS("v_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a0); VOPS("v_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_cvt_pk_bf16_f32 %2, %10, %11\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); }
        if (MODE == 35) { MF(a0); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a0); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\t"); __builtin_amdgcn_sched_barrier(0); }
        if (MODE == 36) { MF(a0); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a0); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_fma_f32 %0, %8, %9, %10\n\tv_exp_f32 %1, %9\n\tv_cvt_pk_bf16_f32 %2, %10, %11\n\t"); __builtin_amdgcn_sched_barrier(0); }
        if (MODE == 37) { MF(a0); VOPS("v_add_f32 %3, %3, %11\n\tv_add_f32 %7, %7, %10\n\tv_add_f32 %3, %3, %11\n\tv_add_f32 %7, %7, %10\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_add_f32 %3, %3, %11\n\tv_add_f32 %7, %7, %10\n\tv_add_f32 %3, %3, %11\n\tv_add_f32 %7, %7, %10\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_add_f32 %3, %3, %11\n\tv_add_f32 %7, %7, %10\n\tv_add_f32 %3, %3, %11\n\tv_add_f32 %7, %7, %10\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_add_f32 %3, %3, %11\n\tv_add_f32 %7, %7, %10\n\tv_add_f32 %3, %3, %11\n\tv_add_f32 %7, %7, %10\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a0); VOPS("v_add_f32 %3, %3, %11\n\tv_add_f32 %7, %7, %10\n\tv_add_f32 %3, %3, %11\n\tv_add_f32 %7, %7, %10\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a1); VOPS("v_add_f32 %3, %3, %11\n\tv_add_f32 %7, %7, %10\n\tv_add_f32 %3, %3, %11\n\tv_add_f32 %7, %7, %10\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a2); VOPS("v_add_f32 %3, %3, %11\n\tv_add_f32 %7, %7, %10\n\tv_add_f32 %3, %3, %11\n\tv_add_f32 %7, %7, %10\n\t"); __builtin_amdgcn_sched_barrier(0); MF(a3); VOPS("v_add_f32 %3, %3, %11\n\tv_add_f32 %7, %7, %10\n\tv_add_f32 %3, %3, %11\n\tv_add_f32 %7, %7, %10\n\t"); __builtin_amdgcn_sched_barrier(0); }
    }
    const uint64_t t1 = memtime(), r1 = realtime();
    float s = y0 + y1 + y2 + y3 + y4 + y5 + y6 + y7 + (float)(p0 + p1 + p2 + p3);
    for (int v = 0; v < 16; ++v) s += a0[v] + a1[v] + a2[v] + a3[v];
    if (s == 12345.678f) out[1000] = 1;
    if ((threadIdx.x & 63) == 0) {
        out[(blockIdx.x * 8 + wave) * 2] = t1 - t0;
        out[(blockIdx.x * 8 + wave) * 2 + 1] = r1 - r0;
    }
}

template <int MODE>
void run(const char *what, int units_per_iter, int grid)
{
    uint64_t *out;
    (void)hipMalloc(&out, 256 * 8 * 2 * 8 + 8192 * 8);
    (void)hipMemset(out, 0, 256 * 8 * 2 * 8 + 8192 * 8);
    const int iters = 2000;
    k<MODE><<<grid, 512>>>(out, 10, 1.0f);
    (void)hipDeviceSynchronize();
    k<MODE><<<grid, 512>>>(out, iters, 1.0f);
    (void)hipDeviceSynchronize();
    uint64_t h[16];
    (void)hipMemcpy(h, out, sizeof(h), hipMemcpyDeviceToHost);
    // wave 0 (group 0) and wave 4 (group 1) of workgroup 0
    const double c0 = (double)h[0] / iters, c4 = (double)h[8] / iters;
    const double us0 = (double)h[1] / 100.0, us4 = (double)h[9] / 100.0;
    printf("mode %2d grid %3d %-58s wave0 %8.1f clk/iter (%6.2f /unit)  wave4 %8.1f (%6.2f /unit)  %.1f us -> %.0f MHz\n", MODE, grid, what, c0,
           c0 / units_per_iter, c4, c4 / units_per_iter, us0, us0 > 0 ? (double)h[0] / us0 : 0.0);
    (void)us4;
    (void)hipFree(out);
}

int main()
{
    for (int grid : {1, 256}) {
        run<0>("32 exp", 32, grid);
        run<1>("32 fma", 32, grid);
        run<2>("32 max3", 32, grid);
        run<3>("32 cvt_pk_bf16", 32, grid);
        run<4>("32 dot2c", 32, grid);
        run<5>("8 mfma", 8, grid);
        run<6>("8 x (mfma + 4 fma)", 8, grid);
        run<7>("8 x (mfma + 6 fma)", 8, grid);
        run<8>("8 x (mfma + 8 fma)", 8, grid);
        run<9>("8 x (mfma + 1 exp)", 8, grid);
        run<10>("8 x (mfma + 2 exp)", 8, grid);
        run<11>("8 x (mfma + fma, exp, cvt, dot)", 8, grid);
        run<12>("g0: 8 mfma | g1: 32 fma", 8, grid);
        run<13>("g0: 8 mfma | g1: 32 exp", 8, grid);
        run<14>("g0: 8 mfma | g1: 8 x (fma, exp, cvt, dot)", 8, grid);
        run<15>("both: 16 mfma, then 16 fma 16 exp 8 cvt 8 dot (lockstep)", 16, grid);
        run<16>("same, groups in opposite order (ping-pong)", 16, grid);
        run<17>("both: 16 x (mfma + fma, exp, cvt, dot) fine interleave", 16, grid);
    }
    // one matrix instruction followed by a few vector instructions, eight times per iteration
    {
        const int grid = 1;
        run<20>("mfma + 4 cvt", 8, grid);
        run<21>("mfma + 4 dot2c", 8, grid);
        run<22>("mfma + 4 max3", 8, grid);
        run<23>("mfma + exp + 3 fma", 8, grid);
        run<24>("mfma + 2 exp + 2 fma", 8, grid);
        run<25>("mfma + fma, exp, cvt, fma", 8, grid);
        run<26>("mfma + fma, exp, fma, dot", 8, grid);
        run<27>("mfma + fma, exp, cvt, add", 8, grid);
        run<28>("mfma + fma, exp, add", 8, grid);
        run<29>("mfma + 1 dot2c", 8, grid);
        run<30>("mfma + 1 cvt", 8, grid);
        run<31>("2 mfma + 2 fma 2 exp 1 cvt 2 add", 8, grid);
        run<32>("2 mfma + 2 fma 2 exp 1 cvt 1 dot", 8, grid);
        run<33>("mfma + 2 dot2c", 8, grid);
        run<34>("mfma + 2 cvt", 8, grid);
        run<35>("mfma + fma, exp", 8, grid);
        run<36>("mfma + fma, exp, cvt", 8, grid);
        run<37>("mfma + 4 add (dependent chain pairs)", 8, grid);
    }
    return 0;
}
