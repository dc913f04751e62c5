// The attention kernel's inner loop on its own (gfx950): per 32-key step and wave 16 matrix
// instructions (8 for the next scores, 8 for P V), the softmax of 16 scores and the LDS operand
// reads, without tile loads, masks or epilogue.  CB = blocks of 32 query rows per wave (1: eight
// waves, two per SIMD; 2: four waves, one per SIMD, every operand read feeds two matrix
// instructions).  Not part of the library; build and run by hand:
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 -Xclang -target-feature -Xclang -packed-fp32-ops \
//       paper_2604_12989_amd/microbench/attn_loop.hip -o /tmp/attn_loop && /tmp/attn_loop
// "/tmp/attn_loop lds" runs the eight-wave loop on 256 workgroups in variants that differ in
// their LDS traffic only -- K operand reads alone, V operand reads alone, both, and both with the
// tile loads of the real kernel (LDS-DMA from a buffer that stays in L2 into a ring of four
// stages, one barrier per tile) -- one kernel name each, for per-kernel counters:
//   rocprofv3 --pmc SQ_LDS_BANK_CONFLICT SQ_ACTIVE_INST_LDS SQ_INSTS_LDS SQ_WAVE_CYCLES -- /tmp/attn_loop lds
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdint>
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
template <int OFF>
__device__ __forceinline__ void lds_rd128(u32x4 &v, uint32_t addr)
{
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "+v"(v) : "v"(addr), "n"(OFF) : "memory");
}
template <int OFF>
__device__ __forceinline__ void lds_rdtr(u32x2 &v, uint32_t addr)
{
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "+v"(v) : "v"(addr), "n"(OFF) : "memory");
}
__device__ __forceinline__ uint32_t f2bf_pair(float lo, float hi)
{
    const floatx2 f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}
template <int N> struct IC { static constexpr int value = N; };
template <int B, int E, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (B < E) { f(IC<B>{}); static_for<B + 1, E>(f); }
}

constexpr int kStage = 17408 + 18432;  // one K tile (64 rows of 272 B) and one V tile (64 rows of 288 B)

// RD: bit 0 = K operand reads, bit 1 = V operand reads.  DMA: the tile loads as well (a ring of
// four stages; needs 4 * kStage bytes of LDS and gsrc, kStage bytes of global memory).
// SWZ: V rows of 256 B without padding, the four 64-byte column blocks of a row stored at
// position (block ^ (row & 3)) -- the layout of the kernel; otherwise rows padded to 288 B.
// STG: the two waves of a SIMD (w and w + 4) issue their tile loads in different halves of the tile.
// VAR (with DMA): 1 = no wait for the loads inside the loop (what the operand reads find is then
// whatever has landed: timing only); 2 = K tiles only; 3 = the loads of a tile are issued by four
// waves, one per SIMD: waves 0-3 for even tiles, 4-7 for odd ones; 4 = all loads of a tile by one
// wave, the eight waves taking turns; 5 = by two waves (w and w + 4 of one SIMD... no: w and w + 1), in turns.
template <int CB, int WAVES, bool BAR, int RD = 3, bool DMA = false, bool SWZ = false, bool STG = false, int VAR = 0>
__global__ __launch_bounds__(64 * WAVES) __attribute__((amdgpu_waves_per_eu(WAVES / 4, WAVES / 4))) void k(float *out, int iters, float scale, uint64_t *cyc, const unsigned char *gsrc = nullptr)
{
    extern __shared__ __align__(16) unsigned char smem[];
    for (int i = threadIdx.x; i < (DMA ? 4 * kStage : 36 * 1024) / 4; i += 64 * WAVES) ((unsigned *)smem)[i] = 0x3c003c00u + (i & 7);
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const unsigned base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    const unsigned ka = base + (lane & 31) * 272 + (lane >> 5) * 16;
    constexpr int VR = SWZ ? 256 : 288;
    const unsigned va = base + 17408 + (4 * (lane >> 5) + ((lane & 15) >> 2)) * VR + 32 * ((lane >> 4) & 1) + 8 * (lane & 3) +
                        (SWZ ? ((lane & 15) >> 2) * 64 : 0);
    floatx16 o[CB][4], sa[CB], sb[CB];
    for (int c = 0; c < CB; ++c) {
        for (int i = 0; i < 4; ++i) for (int v = 0; v < 16; ++v) o[c][i][v] = 0.f;
        for (int v = 0; v < 16; ++v) { sa[c][v] = 0.01f * v; sb[c][v] = 0.02f * v; }
    }
    bf16x8 q[CB][8];
    for (int c = 0; c < CB; ++c)
        for (int ks = 0; ks < 8; ++ks) for (int j = 0; j < 8; ++j) q[c][ks][j] = (__bf16)(0.01f * (threadIdx.x + j + ks + c));
    u32x4 kbuf[8];
    u32x2 vbuf[2][4][2];
    for (int i = 0; i < 8; ++i) kbuf[i] = (u32x4){0x3c003c00u, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u};
    for (int a = 0; a < 2; ++a) for (int b = 0; b < 4; ++b) for (int c = 0; c < 2; ++c) vbuf[a][b][c] = (u32x2){0x3c003c00u, 0x3c003c00u};
    uint32_t pa[CB][8], pb[CB][8];
    for (int c = 0; c < CB; ++c) for (int i = 0; i < 8; ++i) pa[c][i] = pb[c][i] = 0x3c003c00u;
    float lsum[CB];
    for (int c = 0; c < CB; ++c) lsum[c] = 0.f;
    const float mref = 1.0f;
    uint64_t t0;
    asm volatile("s_memtime %0\n\ts_waitcnt lgkmcnt(0)" : "=s"(t0)::"memory");

    auto step = [&](floatx16 (&cur)[CB], floatx16 (&nxt)[CB], uint32_t (&pin)[CB][8], uint32_t (&pout)[CB][8], unsigned ka, unsigned va) __attribute__((always_inline)) {
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        static_for<0, 8>([&](auto I) {
            constexpr int i = decltype(I)::value;
            const bf16x8 a = __builtin_bit_cast(bf16x8, kbuf[i]);
            float e0[CB], e1[CB];
#pragma unroll
            for (int c = 0; c < CB; ++c) {
                if (i == 0) {
                    floatx16 z;
                    for (int v = 0; v < 16; ++v) z[v] = 0.f;
                    nxt[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, q[c][i], z, 0, 0, 0);
                } else {
                    nxt[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, q[c][i], nxt[c], 0, 0, 0);
                }
                if (c == CB - 1 && (RD & 1)) lds_rd128<i * 32>(kbuf[i], ka);
                e0[c] = __builtin_amdgcn_exp2f(fmaf(cur[c][2 * i], scale, -mref));
                lsum[c] += e0[c];
                __builtin_amdgcn_sched_barrier(0);
            }
            constexpr int t2 = i / 4, db = i % 4;
            const bf16x8 va_ = __builtin_bit_cast(bf16x8, (u32x4){vbuf[t2][db][0].x, vbuf[t2][db][0].y, vbuf[t2][db][1].x, vbuf[t2][db][1].y});
#pragma unroll
            for (int c = 0; c < CB; ++c) {
                const bf16x8 pp = __builtin_bit_cast(bf16x8, (u32x4){pin[c][4 * t2], pin[c][4 * t2 + 1], pin[c][4 * t2 + 2], pin[c][4 * t2 + 3]});
                o[c][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va_, pp, o[c][db], 0, 0, 0);
                if (c == CB - 1 && (RD & 2)) {
                    if constexpr (SWZ) {
                        const unsigned vx = va ^ (unsigned)(db * 64);
                        lds_rdtr<(t2 * 16) * 256>(vbuf[t2][db][0], vx);
                        lds_rdtr<(t2 * 16 + 8) * 256>(vbuf[t2][db][1], vx);
                    } else {
                        lds_rdtr<(t2 * 16) * 288 + db * 64>(vbuf[t2][db][0], va);
                        lds_rdtr<(t2 * 16 + 8) * 288 + db * 64>(vbuf[t2][db][1], va);
                    }
                }
                e1[c] = __builtin_amdgcn_exp2f(fmaf(cur[c][2 * i + 1], scale, -mref));
                lsum[c] += e1[c];
                pout[c][i] = f2bf_pair(e0[c], e1[c]);
                __builtin_amdgcn_sched_barrier(0);
            }
        });
    };
    // tile loads as the attention kernel issues them: 17 + 18 blocks of 1 KB per tile, dealt
    // round-robin to the eight waves (4 or 5 loads each), lane l of a block fetching 16 bytes
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    auto issue_tile = [&](int stage) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < (VAR == 4 ? 18 : VAR == 5 ? 9 : VAR == 3 ? 5 : 3); ++i) {
            const int blk = VAR == 4 ? i : VAR == 5 ? 2 * i + (wave & 1) : VAR == 3 ? 4 * i + (wave & 3) : WAVES * i + wave;
            uint32_t off = (uint32_t)(blk * 64 + lane) * 16;
            asm volatile("" : "+v"(off));
            if (blk < 17)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(gsrc + off),
                                                 (__attribute__((address_space(3))) void *)(smem + stage * kStage + blk * 1024), 16, 0, 0);
            if (blk < 18 && VAR != 2)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(gsrc + 17408 + off),
                                                 (__attribute__((address_space(3))) void *)(smem + stage * kStage + 17408 + blk * 1024), 16, 0, 0);
        }
    };
    if (DMA) {
        issue_tile(1);
        issue_tile(2);
    }
    for (int it = 0; it < iters; ++it) {
        if (DMA) {
            // (as in the kernel: everything but the tile requested last has landed, then the barrier)
            if (VAR == 0 || VAR == 2) {
                if (VAR == 2) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
                else if (wave == 0) asm volatile("s_waitcnt vmcnt(5)" ::: "memory");
                else asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
            } else if (VAR == 3) {
                // this wave's previous tile (two iterations back) was its last but one request
                asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
            } else if (VAR >= 4) {
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // (its last request is at least four tiles old)
            }
            __syncthreads();
            if (VAR == 3) {
                if ((wave >> 2) == (it & 1)) issue_tile((it + 3) & 3);
            } else if (VAR == 4) {
                if (wave == (it & 7)) issue_tile((it + 3) & 3);
            } else if (VAR == 5) {
                if ((wave >> 1) == (it & 3)) issue_tile((it + 3) & 3);
            } else if (!STG || wave < 4) issue_tile((it + 3) & 3);
            const unsigned so = (unsigned)(it & 3) * kStage;
            step(sa, sb, pa, pb, ka + so, va + so);
            if (STG && wave >= 4) issue_tile((it + 3) & 3);
            step(sb, sa, pb, pa, ka + so + 32 * 272, va + so + 32 * 288);
        } else {
            step(sa, sb, pa, pb, ka, va);
            step(sb, sa, pb, pa, ka, va);
            if (BAR) __syncthreads();
        }
    }
    if (DMA) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    uint64_t t1;
    asm volatile("s_memtime %0\n\ts_waitcnt lgkmcnt(0)" : "=s"(t1)::"memory");
    float s = 0.f;
    for (int c = 0; c < CB; ++c) {
        s += lsum[c];
        for (int i = 0; i < 4; ++i) for (int v = 0; v < 16; ++v) s += o[c][i][v];
        for (int v = 0; v < 16; ++v) s += sa[c][v] + sb[c][v];
    }
    out[blockIdx.x * 512 + threadIdx.x] = s;
    if ((threadIdx.x & 63) == 0) cyc[blockIdx.x * 8 + (threadIdx.x >> 6)] = t1 - t0;
}

template <int CB, int WAVES, bool BAR>
void run(const char *what, int grid)
{
    float *out; uint64_t *cyc;
    (void)hipMalloc(&out, (size_t)256 * 512 * 4); (void)hipMalloc(&cyc, 256 * 8 * 8);
    (void)hipMemset(cyc, 0, 256 * 8 * 8);
    (void)hipFuncSetAttribute((const void *)k<CB, WAVES, BAR>, hipFuncAttributeMaxDynamicSharedMemorySize, 40 * 1024);
    const int iters = 1000;
    k<CB, WAVES, BAR><<<grid, 64 * WAVES, 40 * 1024>>>(out, 10, 0.125f, cyc);
    (void)hipDeviceSynchronize();
    hipEvent_t e0, e1; (void)hipEventCreate(&e0); (void)hipEventCreate(&e1);
    (void)hipEventRecord(e0);
    k<CB, WAVES, BAR><<<grid, 64 * WAVES, 40 * 1024>>>(out, iters, 0.125f, cyc);
    (void)hipEventRecord(e1);
    (void)hipDeviceSynchronize();
    float ms; (void)hipEventElapsedTime(&ms, e0, e1);
    uint64_t h[8];
    (void)hipMemcpy(h, cyc, sizeof(h), hipMemcpyDeviceToHost);
    uint64_t mx = 0; for (int i = 0; i < WAVES; ++i) mx = h[i] > mx ? h[i] : mx;
    const double mfma_per_simd = 2.0 * 16 * CB * (WAVES / 4);  // per iteration
    printf("%-40s grid %3d: %7.1f clk/iter = %5.1f clk per MFMA of a SIMD; %.3f ms -> %4.0f TFLOP/s at %.0f MHz\n", what, grid,
           (double)mx / iters, (double)mx / iters / mfma_per_simd, ms, (double)iters * mfma_per_simd * 4 * grid * 32768.0 / ms / 1e9,
           (double)mx / (ms * 1e3));
    (void)hipFree(out); (void)hipFree(cyc);
}
// The eight-wave loop on 256 workgroups with K reads, V reads, both, and both plus tile loads.
template <int RD, bool DMA, bool SWZ = false, bool STG = false, int VAR = 0>
void run_lds(const char *what)
{
    float *out; uint64_t *cyc; unsigned char *gsrc;
    (void)hipMalloc(&out, (size_t)256 * 512 * 4); (void)hipMalloc(&cyc, 256 * 8 * 8); (void)hipMalloc(&gsrc, kStage);
    (void)hipMemset(gsrc, 0x3c, kStage);
    const int lds = DMA ? 4 * kStage : 40 * 1024, iters = 1000;
    (void)hipFuncSetAttribute((const void *)k<1, 8, true, RD, DMA, SWZ, STG, VAR>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    k<1, 8, true, RD, DMA, SWZ, STG, VAR><<<256, 512, lds>>>(out, 10, 0.125f, cyc, gsrc);
    (void)hipDeviceSynchronize();
    k<1, 8, true, RD, DMA, SWZ, STG, VAR><<<256, 512, lds>>>(out, iters, 0.125f, cyc, gsrc);
    (void)hipDeviceSynchronize();
    uint64_t h[8];
    (void)hipMemcpy(h, cyc, sizeof(h), hipMemcpyDeviceToHost);
    uint64_t mx = 0; for (int i = 0; i < 8; ++i) mx = h[i] > mx ? h[i] : mx;
    printf("%-44s %7.1f clk per 64-key tile (workgroup 0)\n", what, (double)mx / iters);
    (void)hipFree(out); (void)hipFree(cyc); (void)hipFree(gsrc);
}
int main(int argc, char **argv)
{
    if (argc > 1 && argv[1][0] == 'l') {
        run_lds<1, false>("K operand reads only");
        run_lds<2, false>("V operand reads only");
        run_lds<3, false>("K and V operand reads");
        run_lds<3, true>("K and V operand reads + tile loads (LDS-DMA)");
        run_lds<0, true>("tile loads only");
        run_lds<2, false, true>("V operand reads only, swizzled rows of 256 B");
        run_lds<3, false, true>("K and V operand reads, V swizzled");
        run_lds<3, true, false, true>("K and V reads + tile loads, the waves of a SIMD staggered");
        run_lds<3, true, false, false, 1>("K and V reads + tile loads, no wait for the loads");
        run_lds<3, true, false, false, 2>("K and V reads + K tile loads only");
        run_lds<3, true, false, false, 3>("K and V reads + tile loads by one wave per SIMD, alternating");
        run_lds<3, true, false, false, 4>("K and V reads + tile loads by one wave, in turns");
        run_lds<3, true, false, false, 5>("K and V reads + tile loads by two waves, in turns");
        return 0;
    }
    for (int grid : {1, 256}) {
        run<1, 8, true>("CB=1, 8 waves, barrier per tile", grid);
        run<1, 8, false>("CB=1, 8 waves, no barrier", grid);
        run<1, 4, true>("CB=1, 4 waves, barrier per tile", grid);
        run<2, 4, true>("CB=2, 4 waves, barrier per tile", grid);
        run<2, 4, false>("CB=2, 4 waves, no barrier", grid);
    }
    return 0;
}
