// Tree attention for the verifier pass (paper Section 4.4, first paragraph): every tree node
// attends to the whole cached context and, inside the tree, only to the root, its ancestors and
// itself (the ancestor bitmask).
//
// Two device paths behind ddtree_verify_attn:
//   * attn_mfma_kernel   bf16, head_dim 128: flash-style kernel on the gfx950 matrix cores.
//   * attn_generic_kernel  any supported shape and fp32: one workgroup per (node, head) on the
//                        vector ALUs; used for the small fp32 configuration and odd shapes.
//
// MFMA kernel.  Query rows of one KV head are the (node, group-head) pairs, G = Hq/Hkv per node,
// so one K/V tile serves G*T rows.  A workgroup (4 waves) owns 256 consecutive rows (64 per
// wave) and a contiguous range of 64-key tiles (split-KV; partial results are merged by
// attn_merge_kernel).  Per tile:
//   S^T = K Q^T   v_mfma_f32_32x32x16_bf16, A = K tile from LDS (row = key), B = Q^T held in
//                 registers for the whole kernel.  In the accumulator layout a lane then owns
//                 one query row, so the softmax max and sum are register-local reductions.
//   P^T           exp2 of the scaled, masked scores; the accumulator registers of S^T are, as
//                 they stand, the B operand of the next product (no cross-lane movement).
//   O^T += V^T P^T  A = V^T, gathered from the row-major V tile in LDS by the transposing
//                 LDS read, in the key order the P^T registers happen to have.
// The running maximum is a lagging reference: accumulators are rescaled only when a row's
// maximum grows by more than 2^8, so the steady state has no rescale work at all.
// K and V tiles sit in LDS as [key][dim], rows padded (272 B / 288 B) so that the 16-byte K
// reads and the transposing V reads are free of bank conflicts.
// The ancestor mask touches only the tree tiles (the last ceil(T/64) tiles): one 64-bit word per
// (row, tile), bit test per score.  Cache tiles carry no mask work at all.
#include "common.hpp"

namespace ddt {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int kAttnThreads = 256;
constexpr int kMT = 256;       // query rows per workgroup
constexpr int kKT = 64;        // keys per tile
constexpr int kHD = 128;       // head dim of the MFMA path
constexpr int kKStride = kHD + 8;   // bf16 elements per K row in LDS (272 B)
constexpr int kVStride = kHD + 16;  // bf16 elements per V row in LDS (288 B)
constexpr float kLog2e = 1.4426950408889634f;
constexpr int kAttnStages = 2;
constexpr int kAttnLdsBytes = kAttnStages * 2 * kKT * kHD * 2;  // stages x {K, V} x 16 KB

struct AttnArgs {
    int32_t kv_offset[DDTREE_MAX_BATCH + 1];
};

AttnPlan attn_plan(int batch, int T, int Hq, int Hkv, int D, long long sum_L, int dtype)
{
    AttnPlan p{};
    p.splits = 1;
    p.mtiles = 0;
    p.bytes = 0;
    if (!(dtype == DDTREE_DTYPE_BF16 && D == kHD)) return p;  // generic path needs no scratch
    const int G = Hq / Hkv;
    const long long M = (long long)T * G;
    p.mtiles = (int)((M + kMT - 1) / kMT);
    const long long full = M / kMT > 0 ? M / kMT : 1;
    const long long base = (long long)batch * Hkv * full;
    int S;
    if (base >= 512) S = 1;
    else if (base >= 256) S = 2;
    else S = (int)((256 + base - 1) / base);
    // keep at least four tiles per split on average
    const long long tiles = (sum_L / batch + T) / kKT;
    if ((long long)S * 4 > tiles) S = (int)(tiles / 4 > 0 ? tiles / 4 : 1);
    if (S > 32) S = 32;
    p.splits = S;
    if (S > 1) {
        const size_t rows = (size_t)batch * T * Hq;
        p.part_off = 0;
        p.lse_off = align_up((size_t)S * rows * D * 4, 256);
        p.bytes = align_up(p.lse_off + (size_t)S * rows * 4, 256);
    }
    return p;
}

// Upper bound of attn_plan(...).bytes over all sum_L: splits only shrink with shorter caches.
size_t attn_ws_upper(int batch, int T, int Hq, int Hkv, int D)
{
    AttnPlan p = attn_plan(batch, T, Hq, Hkv, D, (long long)1 << 40, DDTREE_DTYPE_BF16);
    return p.bytes;
}

__device__ __forceinline__ uint32_t pack_lo(uint32_t a, uint32_t b) { return (a & 0xFFFFu) | (b << 16); }
__device__ __forceinline__ uint32_t pack_hi(uint32_t a, uint32_t b) { return (a >> 16) | (b & 0xFFFF0000u); }
__device__ __forceinline__ uint32_t f2bf_pair(float lo, float hi)
{
    const __bf16 a = (__bf16)lo, b = (__bf16)hi;
    return (uint32_t)__builtin_bit_cast(unsigned short, a) |
           ((uint32_t)__builtin_bit_cast(unsigned short, b) << 16);
}

// Reads of the K/V tiles are written as asm.  The tiles are filled by LDS-DMA
// (global_load_lds); the compiler cannot tell which stage a given LDS read touches and would
// wait for every outstanding tile load before each read, serialising prefetch and compute.  With
// asm reads the waits are placed by hand: s_waitcnt vmcnt(0) + barrier once per tile for the
// DMA, lds_wait() below for the reads.
__device__ __forceinline__ u32x4 lds_rd128(uint32_t addr)
{
    u32x4 v;
    asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(addr) : "memory");
    return v;
}
__device__ __forceinline__ u32x4 lds_rd128_8k(uint32_t addr)
{
    u32x4 v;
    asm volatile("ds_read_b128 %0, %1 offset:8192" : "=v"(v) : "v"(addr) : "memory");
    return v;
}
// LDS transpose read (ds_read_b64_tr_b16).  Within each group of 16 lanes, lane 4*j + r points
// at four consecutive 16-bit elements; afterwards lane i of the group holds, for j = 0..3, element
// i % 4 of what lane 4*j + i / 4 pointed at.  With lane 4*j + r pointing at V[key_j][d0 + 4*r ..],
// lane i receives V[key_0..3][d0 + i]: a column of the row-major V tile, which is what the A
// operand (V^T) of the second product needs.
__device__ __forceinline__ u32x2 lds_rdtr(uint32_t addr)
{
    u32x2 v;
    asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(v) : "v"(addr) : "memory");
    return v;
}
__device__ __forceinline__ u32x2 lds_rdtr_2k(uint32_t addr)
{
    u32x2 v;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:2048" : "=v"(v) : "v"(addr) : "memory");
    return v;
}
// Wait until every LDS read issued so far has returned; the operands tie the wait to the
// registers it protects so that their uses cannot be scheduled above it.
__device__ __forceinline__ void lds_wait(u32x4 &a, u32x4 &b)
{
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a), "+v"(b) : : "memory");
}
__device__ __forceinline__ void lds_wait8(u32x2 (&v)[4][2])
{
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(v[0][0]), "+v"(v[0][1]), "+v"(v[1][0]), "+v"(v[1][1]), "+v"(v[2][0]),
                   "+v"(v[2][1]), "+v"(v[3][0]), "+v"(v[3][1])
                 :
                 : "memory");
}

// acc *= alpha when flag != 0 (flag is wave-uniform), in place in the accumulator registers.
// The branch lives inside the asm so that, for the compiler, the accumulators flow straight
// through: a C++ "if" around a VALU update makes it keep a second copy of all of them.
__device__ __forceinline__ void scale_acc_if(floatx16 &acc, float alpha, int flag)
{
    float e0 = acc[0], e1 = acc[1], e2 = acc[2], e3 = acc[3], e4 = acc[4], e5 = acc[5], e6 = acc[6],
          e7 = acc[7], e8 = acc[8], e9 = acc[9], e10 = acc[10], e11 = acc[11], e12 = acc[12],
          e13 = acc[13], e14 = acc[14], e15 = acc[15];
    float tmp;
#define DDT_SC(n) "v_accvgpr_read_b32 %16, %" #n "\n\ts_nop 0\n\tv_mul_f32 %16, %16, %17\n\ts_nop 0\n\tv_accvgpr_write_b32 %" #n ", %16\n\t"
    asm volatile("s_cmp_eq_u32 %18, 0\n\t"
                 "s_cbranch_scc1 ddt_skip_%=\n\t"
                 "s_nop 15\n\ts_nop 7\n\t"  // let matrix results land before reading them
                 DDT_SC(0) DDT_SC(1) DDT_SC(2) DDT_SC(3) DDT_SC(4) DDT_SC(5) DDT_SC(6) DDT_SC(7)
                 DDT_SC(8) DDT_SC(9) DDT_SC(10) DDT_SC(11) DDT_SC(12) DDT_SC(13) DDT_SC(14) DDT_SC(15)
                 "s_nop 7\n"
                 "ddt_skip_%=:"
                 : "+a"(e0), "+a"(e1), "+a"(e2), "+a"(e3), "+a"(e4), "+a"(e5), "+a"(e6), "+a"(e7),
                   "+a"(e8), "+a"(e9), "+a"(e10), "+a"(e11), "+a"(e12), "+a"(e13), "+a"(e14),
                   "+a"(e15), "=&v"(tmp)
                 : "v"(alpha), "s"(__builtin_amdgcn_readfirstlane(flag))
                 : "scc");
#undef DDT_SC
    acc[0] = e0; acc[1] = e1; acc[2] = e2; acc[3] = e3; acc[4] = e4; acc[5] = e5; acc[6] = e6;
    acc[7] = e7; acc[8] = e8; acc[9] = e9; acc[10] = e10; acc[11] = e11; acc[12] = e12;
    acc[13] = e13; acc[14] = e14; acc[15] = e15;
}

constexpr float kRescaleThreshold = 8.0f;  // log2 units: stale running max tolerated up to 2^8

__global__ __launch_bounds__(kAttnThreads) __attribute__((amdgpu_waves_per_eu(1, 1)))
void attn_mfma_kernel(const uint16_t *__restrict__ q, const uint16_t *__restrict__ k_cache,
                      const uint16_t *__restrict__ v_cache, const uint16_t *__restrict__ k_tree,
                      const uint16_t *__restrict__ v_tree, const uint64_t *__restrict__ mask,
                      AttnArgs args, int T, int Hq, int Hkv, float scale_log2e, int splits,
                      uint16_t *__restrict__ out, float *__restrict__ part, float *__restrict__ part_lse)
{
    // LDS: kStages stages of {K tile, V tile}, each tile 64 keys x 256 B, filled by direct
    // global->LDS loads (64 lanes x 16 B land contiguously, so a wave instruction fills 4 rows).
    // Bank conflicts are avoided by swizzling the 16-byte column index per row: K stores column c
    // of key r at position c ^ (r & 7), V at position c ^ (2 * (r & 3)).
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int kTileBytes = kKT * kHD * 2;      // 16 KB
    constexpr int kStageBytes = 2 * kTileBytes;    // K then V

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int split = blockIdx.x;
    const int hk = blockIdx.y % Hkv, mt = blockIdx.y / Hkv;
    const int seq = blockIdx.z;
    const int G = Hq / Hkv;
    const int W = (T + 63) >> 6;
    const int M = T * G;
    const int L0 = args.kv_offset[seq];
    const int L = args.kv_offset[seq + 1] - L0;
    const int m0 = mt * kMT;
    const int last_node = min(T - 1, (m0 + kMT - 1) / G);
    const int n_cache_tiles = (L + kKT - 1) / kKT;
    const int n_tree_tiles = last_node / kKT + 1;
    const int nt = n_cache_tiles + n_tree_tiles;
    const int t_begin = (int)((long long)nt * split / splits);
    const int t_end = (int)((long long)nt * (split + 1) / splits);
    const bool wave_active = m0 + wave * 64 < M;

    // this lane's two query rows (cb = 0, 1)
    int node_[2], rowg_[2];
    bool rvalid[2];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        const int r = m0 + wave * 64 + cb * 32 + l32;
        rvalid[cb] = r < M;
        const int node = rvalid[cb] ? r / G : 0;
        const int g = rvalid[cb] ? r - node * G : 0;
        node_[cb] = node;
        rowg_[cb] = (seq * T + node) * Hq + hk * G + g;
    }
    // Q^T operand: lane holds Q[row][16*ks + 8*half .. +8]
    bf16x8 qreg[2][8];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (rvalid[cb])
                v = *reinterpret_cast<const uint4 *>(q + (size_t)rowg_[cb] * kHD + ks * 16 + half * 8);
            qreg[cb][ks] = __builtin_bit_cast(bf16x8, v);
            // the query operand is only ever read by MFMA: park it in the accumulator file
            asm volatile("" : "+a"(qreg[cb][ks]));
        }

    floatx16 o[4][2];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[db][cb][v] = 0.0f;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) asm volatile("" : "+a"(o[db][cb]));
    float m_run[2] = {-INFINITY, -INFINITY};  // reference maximum (may lag the true one)
    float l_run[2] = {0.0f, 0.0f};

    // ---- tile loads: wave w, instruction i fills rows 4*(4*i + w) .. +3 of the K and V tiles;
    //      lane -> (row in block = lane / 16, position = lane % 16) ----
    const size_t rs = (size_t)Hkv * kHD;  // elements between consecutive keys in global memory
    const int ld_r4 = lane >> 4, ld_pos = lane & 15;
    auto issue_tile = [&](int tt, int stage) {
        const uint16_t *kp, *vp;
        int valid_;
        if (tt < n_cache_tiles) {
            const size_t row0 = (size_t)L0 + (size_t)tt * kKT;
            kp = k_cache + (row0 * Hkv + hk) * kHD;
            vp = v_cache + (row0 * Hkv + hk) * kHD;
            valid_ = min(kKT, L - tt * kKT);
        } else {
            const size_t row0 = (size_t)seq * T + (size_t)(tt - n_cache_tiles) * kKT;
            kp = k_tree + (row0 * Hkv + hk) * kHD;
            vp = v_tree + (row0 * Hkv + hk) * kHD;
            valid_ = min(kKT, T - (tt - n_cache_tiles) * kKT);
        }
        unsigned char *st = smem + stage * kStageBytes;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int blk = 4 * i + wave;
            const int r = 4 * blk + ld_r4;
            const int rsrc = min(r, valid_ - 1);  // rows past the end re-read a valid row (finite data)
            const int ck = ld_pos ^ (r & 7);
            const int cv = ld_pos ^ (2 * (r & 3));
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void *)(kp + rsrc * rs + ck * 8),
                (__attribute__((address_space(3))) void *)(st + blk * 1024), 16, 0, 0);
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void *)(vp + rsrc * rs + cv * 8),
                (__attribute__((address_space(3))) void *)(st + kTileBytes + blk * 1024), 16, 0, 0);
        }
    };

    // per-lane LDS read offsets (bytes, relative to the tile), one per compile-time column group
    int k_off[8];  // K: row l32 (+32*kb), column 2*ks + half
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) k_off[ks] = l32 * 256 + (((2 * ks + half) ^ (l32 & 7)) << 4);
    const int lm = lane & 15, dim16 = (lane >> 4) & 1;
    const int vj = lm >> 2, vr = lm & 3;
    int v_off[4];  // V: row 4*half + vj (+16*kstep, +8), column 4*db + 2*dim16 + vr/2, 8-byte half vr%2
#pragma unroll
    for (int db = 0; db < 4; ++db)
        v_off[db] = (4 * half + vj) * 256 + (((4 * db + 2 * dim16 + (vr >> 1)) ^ (2 * vj)) << 4) + 8 * (vr & 1);

    const uint32_t lds_base =
        (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;

    if (t_begin < t_end) issue_tile(t_begin, 0);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    for (int t = t_begin; t < t_end; ++t) {
        const int stage = (t - t_begin) & 1;
        if (t + 1 < t_end) issue_tile(t + 1, stage ^ 1);
        if (wave_active) {
        const uint32_t sK_addr = lds_base + stage * kStageBytes;
        const uint32_t sV_addr = sK_addr + kTileBytes;

        const bool is_tree = t >= n_cache_tiles;
        const int tb = t - n_cache_tiles;
        const int valid = is_tree ? min(kKT, T - tb * kKT) : min(kKT, L - t * kKT);

        // ---- S^T = K Q^T ----
        floatx16 s[2][2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int cb = 0; cb < 2; ++cb)
#pragma unroll
                for (int v = 0; v < 16; ++v) s[kb][cb][v] = 0.0f;
        {
            u32x4 ka[2][2];  // [buffer][kb]: operands of k-step ks + 1 are in flight during step ks
            ka[0][0] = lds_rd128(sK_addr + k_off[0]);
            ka[0][1] = lds_rd128_8k(sK_addr + k_off[0]);
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const int cur = ks & 1;
                lds_wait(ka[cur][0], ka[cur][1]);
                if (ks + 1 < 8) {
                    ka[cur ^ 1][0] = lds_rd128(sK_addr + k_off[ks + 1]);
                    ka[cur ^ 1][1] = lds_rd128_8k(sK_addr + k_off[ks + 1]);
                }
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    const bf16x8 a = __builtin_bit_cast(bf16x8, ka[cur][kb]);
#pragma unroll
                    for (int cb = 0; cb < 2; ++cb)
                        s[kb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[cb][ks], s[kb][cb], 0, 0, 0);
                }
            }
        }

        // ---- mask (tree tiles and a ragged last cache tile only) ----
        if (is_tree || valid < kKT) {
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) {
                uint64_t word = ~0ull;
                if (is_tree)
                    word = rvalid[cb] ? mask[((size_t)seq * T + node_[cb]) * W + tb] : 0ull;
                if (valid < kKT) word &= (1ull << valid) - 1ull;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int key = kb * 32 + (v >> 2) * 8 + half * 4 + (v & 3);
                        if (!((word >> key) & 1ull)) s[kb][cb][v] = -INFINITY;
                    }
            }
        }

        // ---- online softmax, one query row per lane and cb, lazily rescaled ----
        float m_new[2];
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            float tmax = s[0][cb][0];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) tmax = fmaxf(tmax, s[kb][cb][v]);
            tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
            m_new[cb] = fmaxf(m_run[cb], tmax * scale_log2e);
        }
        // The running reference is only moved when some row's maximum grew by more than the
        // threshold (always the case on a row's first visible key); otherwise exp2 arguments
        // stay below the threshold and nothing has to be rescaled.
        const int resc = __any((m_new[0] > m_run[0] + kRescaleThreshold) |
                               (m_new[1] > m_run[1] + kRescaleThreshold));
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            const float m_tgt = resc ? m_new[cb] : m_run[cb];
            const float m_use = m_tgt == -INFINITY ? 0.0f : m_tgt;
            const float alpha = __builtin_amdgcn_exp2f(m_run[cb] - m_use);  // exactly 1 when kept
            m_run[cb] = m_tgt;
            l_run[cb] *= alpha;
#pragma unroll
            for (int db = 0; db < 4; ++db) scale_acc_if(o[db][cb], alpha, resc);
        }
        bf16x8 pb[2][4];
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            const float m_use = m_run[cb] == -INFINITY ? 0.0f : m_run[cb];
            float psum = 0.0f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float p = __builtin_amdgcn_exp2f(fmaf(s[kb][cb][v], scale_log2e, -m_use));
                    s[kb][cb][v] = p;
                    psum += p;
                }
#pragma unroll
                for (int t2 = 0; t2 < 2; ++t2) {
                    uint4 pk;
                    pk.x = f2bf_pair(s[kb][cb][8 * t2 + 0], s[kb][cb][8 * t2 + 1]);
                    pk.y = f2bf_pair(s[kb][cb][8 * t2 + 2], s[kb][cb][8 * t2 + 3]);
                    pk.z = f2bf_pair(s[kb][cb][8 * t2 + 4], s[kb][cb][8 * t2 + 5]);
                    pk.w = f2bf_pair(s[kb][cb][8 * t2 + 6], s[kb][cb][8 * t2 + 7]);
                    pb[cb][kb * 2 + t2] = __builtin_bit_cast(bf16x8, pk);
                }
            }
            l_run[cb] += psum;
        }

        // ---- O^T += V^T P^T.  Element j of the P^T operand of k-step kst is key
        //      16*kst + 8*(j/4) + 4*half + j%4; the two transpose reads fetch exactly those keys ----
        {
            u32x2 va[2][4][2];  // [buffer][db][low / high four keys]
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                va[0][db][0] = lds_rdtr(sV_addr + v_off[db]);
                va[0][db][1] = lds_rdtr_2k(sV_addr + v_off[db]);
            }
#pragma unroll
            for (int kst4 = 0; kst4 < 4; ++kst4) {
                const int cur = kst4 & 1;
                lds_wait8(va[cur]);
                if (kst4 + 1 < 4) {
#pragma unroll
                    for (int db = 0; db < 4; ++db) {
                        va[cur ^ 1][db][0] = lds_rdtr(sV_addr + v_off[db] + (kst4 + 1) * 4096);
                        va[cur ^ 1][db][1] = lds_rdtr_2k(sV_addr + v_off[db] + (kst4 + 1) * 4096);
                    }
                }
#pragma unroll
                for (int db = 0; db < 4; ++db) {
                    const bf16x8 a = __builtin_bit_cast(
                        bf16x8, (u32x4){va[cur][db][0].x, va[cur][db][0].y, va[cur][db][1].x, va[cur][db][1].y});
#pragma unroll
                    for (int cb = 0; cb < 2; ++cb)
                        o[db][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[cb][kst4], o[db][cb], 0, 0, 0);
                }
            }
        }
        }
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
    }

    if (!wave_active) return;
    // ---- epilogue ----
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        const float l_tot = l_run[cb] + __shfl_xor(l_run[cb], 32, 64);
        if (!rvalid[cb]) continue;
        const int node = node_[cb];
        const bool real = (mask[((size_t)seq * T + node) * W + (node >> 6)] >> (node & 63)) & 1ull;
        const float inv = (real && l_tot > 0.0f) ? 1.0f / l_tot : 0.0f;
        if (splits == 1) {
            uint16_t *dst = out + (size_t)rowg_[cb] * kHD;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    const int dim = db * 32 + g4 * 8 + half * 4;
                    uint2 val;
                    val.x = f2bf_pair(o[db][cb][4 * g4 + 0] * inv, o[db][cb][4 * g4 + 1] * inv);
                    val.y = f2bf_pair(o[db][cb][4 * g4 + 2] * inv, o[db][cb][4 * g4 + 3] * inv);
                    *reinterpret_cast<uint2 *>(dst + dim) = val;
                }
        } else {
            const size_t rows_total = (size_t)gridDim.z * T * Hq;
            float *dst = part + ((size_t)split * rows_total + rowg_[cb]) * kHD;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    const int dim = db * 32 + g4 * 8 + half * 4;
                    float4 val;
                    val.x = o[db][cb][4 * g4 + 0] * inv;
                    val.y = o[db][cb][4 * g4 + 1] * inv;
                    val.z = o[db][cb][4 * g4 + 2] * inv;
                    val.w = o[db][cb][4 * g4 + 3] * inv;
                    *reinterpret_cast<float4 *>(dst + dim) = val;
                }
            if (half == 0)
                part_lse[(size_t)split * rows_total + rowg_[cb]] =
                    inv > 0.0f ? m_run[cb] + __builtin_amdgcn_logf(l_tot) : -INFINITY;
        }
    }
}

// Merge of the split-KV partials: out = sum_s 2^(lse_s - max) O_s / sum_s 2^(lse_s - max).
__global__ __launch_bounds__(256) void attn_merge_kernel(const float *__restrict__ part,
                                                         const float *__restrict__ part_lse,
                                                         int splits, size_t rows_total,
                                                         uint16_t *__restrict__ out)
{
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;  // (row, 4-dim group)
    const size_t row = idx / (kHD / 4);
    const int dg = (int)(idx % (kHD / 4));
    if (row >= rows_total) return;
    float mx = -INFINITY;
    for (int s = 0; s < splits; ++s) mx = fmaxf(mx, part_lse[(size_t)s * rows_total + row]);
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float wsum = 0.0f;
    if (mx > -INFINITY) {
        for (int s = 0; s < splits; ++s) {
            const float w = __builtin_amdgcn_exp2f(part_lse[(size_t)s * rows_total + row] - mx);
            const float4 v =
                *reinterpret_cast<const float4 *>(part + ((size_t)s * rows_total + row) * kHD + dg * 4);
            acc.x += w * v.x;
            acc.y += w * v.y;
            acc.z += w * v.z;
            acc.w += w * v.w;
            wsum += w;
        }
    }
    const float inv = wsum > 0.0f ? 1.0f / wsum : 0.0f;
    uint2 val;
    val.x = f2bf_pair(acc.x * inv, acc.y * inv);
    val.y = f2bf_pair(acc.z * inv, acc.w * inv);
    *reinterpret_cast<uint2 *>(out + row * kHD + dg * 4) = val;
}

// ------------------------------------------------------------------------------------------
// Generic path: one workgroup per (node, query head); keys in tiles of 256, online softmax,
// fp32 arithmetic with accurate expf.  IO type TIO is float or bf16 bits (uint16_t).
// ------------------------------------------------------------------------------------------
constexpr int kGenThreads = 256;

__device__ __forceinline__ float ld_elem(const float *p) { return *p; }
__device__ __forceinline__ float ld_elem(const uint16_t *p)
{
    return __uint_as_float((uint32_t)(*p) << 16);
}
__device__ __forceinline__ void st_elem(float *p, float v) { *p = v; }
__device__ __forceinline__ void st_elem(uint16_t *p, float v)
{
    const __bf16 b = (__bf16)v;
    *p = __builtin_bit_cast(unsigned short, b);
}

template <typename TIO>
__global__ __launch_bounds__(kGenThreads) void attn_generic_kernel(
    const TIO *__restrict__ q, const TIO *__restrict__ k_cache, const TIO *__restrict__ v_cache,
    const TIO *__restrict__ k_tree, const TIO *__restrict__ v_tree,
    const uint64_t *__restrict__ mask, AttnArgs args, int T, int Hq, int Hkv, int D, float scale,
    TIO *__restrict__ out)
{
    __shared__ float s_q[256];
    __shared__ float s_p[kGenThreads];
    __shared__ float s_red[kGenThreads / 64];
    const int tid = threadIdx.x;
    const int h = blockIdx.x, i = blockIdx.y, seq = blockIdx.z;
    const int G = Hq / Hkv, hk = h / G;
    const int W = (T + 63) >> 6;
    const int L0 = args.kv_offset[seq];
    const int L = args.kv_offset[seq + 1] - L0;
    const size_t qrow = ((size_t)seq * T + i) * Hq + h;
    const uint64_t *mrow = mask + ((size_t)seq * T + i) * W;
    TIO *orow = out + qrow * D;
    const bool real = (mrow[i >> 6] >> (i & 63)) & 1ull;
    if (!real) {
        if (tid < D) st_elem(orow + tid, 0.0f);
        return;
    }
    if (tid < D) s_q[tid] = ld_elem(q + qrow * D + tid);
    __syncthreads();
    float m_run = -INFINITY, l_run = 0.0f, acc = 0.0f;
    const int total = L + T;
    for (int j0 = 0; j0 < total; j0 += kGenThreads) {
        const int j = j0 + tid;
        float s = -INFINITY;
        const TIO *krow = nullptr;
        if (j < L) {
            krow = k_cache + ((size_t)(L0 + j) * Hkv + hk) * D;
        } else if (j < total) {
            const int jt = j - L;
            if ((mrow[jt >> 6] >> (jt & 63)) & 1ull)
                krow = k_tree + (((size_t)seq * T + jt) * Hkv + hk) * D;
        }
        if (krow) {
            float dot = 0.0f;
            for (int c = 0; c < D; ++c) dot = fmaf(s_q[c], ld_elem(krow + c), dot);
            s = dot * scale;
        }
        // tile max
        float tmax = s;
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) tmax = fmaxf(tmax, __shfl_xor(tmax, d, 64));
        if ((tid & 63) == 0) s_red[tid >> 6] = tmax;
        __syncthreads();
        tmax = fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3]));
        __syncthreads();
        const float m_new = fmaxf(m_run, tmax);
        if (m_new == -INFINITY) continue;  // nothing visible yet (uniform across the workgroup)
        const float alpha = expf(m_run - m_new);
        const float p = s == -INFINITY ? 0.0f : expf(s - m_new);
        s_p[tid] = p;
        float psum = p;
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) psum += __shfl_xor(psum, d, 64);
        if ((tid & 63) == 0) s_red[tid >> 6] = psum;
        __syncthreads();
        psum = (s_red[0] + s_red[1]) + (s_red[2] + s_red[3]);
        l_run = l_run * alpha + psum;
        m_run = m_new;
        if (tid < D) {
            acc *= alpha;
            const int cnt = min(kGenThreads, total - j0);
            for (int t = 0; t < cnt; ++t) {
                const float pt = s_p[t];
                if (pt == 0.0f) continue;
                const int jj = j0 + t;
                const TIO *vrow = jj < L ? v_cache + ((size_t)(L0 + jj) * Hkv + hk) * D
                                         : v_tree + (((size_t)seq * T + (jj - L)) * Hkv + hk) * D;
                acc = fmaf(pt, ld_elem(vrow + tid), acc);
            }
        }
        __syncthreads();
    }
    if (tid < D) st_elem(orow + tid, l_run > 0.0f ? acc / l_run : 0.0f);
}

}  // namespace ddt

extern "C" int ddtree_verify_attn(const void *q, const void *k_cache, const void *v_cache,
                                  const void *k_tree, const void *v_tree,
                                  const uint64_t *ancestor_mask, const int32_t *kv_offset, int batch,
                                  int T, int Hq, int Hkv, int D, float softmax_scale, int dtype,
                                  void *out, void *workspace, size_t workspace_bytes, void *stream)
{
    using namespace ddt;
    if (!q || !k_tree || !v_tree || !ancestor_mask || !kv_offset || !out) return DDTREE_ERR_ARG;
    if (batch < 1 || batch > DDTREE_MAX_BATCH || T < 1 || T > DDTREE_MAX_N + 1 || Hq < 1 || Hkv < 1 ||
        Hq % Hkv != 0 || D < 8 || D > 256 || D % 8 != 0)
        return DDTREE_ERR_ARG;
    if (dtype != DDTREE_DTYPE_BF16 && dtype != DDTREE_DTYPE_FP32) return DDTREE_ERR_ARG;
    if (!(softmax_scale > 0.0f) || !(softmax_scale < 1e30f)) return DDTREE_ERR_ARG;
    AttnArgs args;
    if (kv_offset[0] < 0) return DDTREE_ERR_ARG;
    for (int s = 0; s <= batch; ++s) {
        if (s > 0 && kv_offset[s] < kv_offset[s - 1]) return DDTREE_ERR_ARG;
        args.kv_offset[s] = kv_offset[s];
    }
    const long long sum_L = (long long)kv_offset[batch] - kv_offset[0];
    if (kv_offset[batch] > 0 && (!k_cache || !v_cache)) return DDTREE_ERR_ARG;
    hipStream_t st = as_stream(stream);

    if (dtype == DDTREE_DTYPE_BF16 && D == kHD) {
        AttnPlan p = attn_plan(batch, T, Hq, Hkv, D, sum_L, dtype);
        if (!ws_ok(workspace, workspace_bytes, p.bytes)) return DDTREE_ERR_WORKSPACE;
        float *part = p.splits > 1 ? reinterpret_cast<float *>(static_cast<char *>(workspace) + p.part_off) : nullptr;
        float *lse = p.splits > 1 ? reinterpret_cast<float *>(static_cast<char *>(workspace) + p.lse_off) : nullptr;
        static bool attr_set = false;
        if (!attr_set) {
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(attn_mfma_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kAttnLdsBytes) != hipSuccess)
                return DDTREE_ERR_HIP;
            attr_set = true;
        }
        DDT_LAUNCH(DDTREE_KERNEL_ATTN, st, attn_mfma_kernel, dim3(p.splits, p.mtiles * Hkv, batch), dim3(kAttnThreads),
                           kAttnLdsBytes, st, static_cast<const uint16_t *>(q), static_cast<const uint16_t *>(k_cache),
                           static_cast<const uint16_t *>(v_cache), static_cast<const uint16_t *>(k_tree),
                           static_cast<const uint16_t *>(v_tree), ancestor_mask, args, T, Hq, Hkv,
                           softmax_scale * kLog2e, p.splits, static_cast<uint16_t *>(out), part, lse);
        if (p.splits > 1) {
            const size_t rows = (size_t)batch * T * Hq;
            const size_t threads = rows * (kHD / 4);
            DDT_LAUNCH(DDTREE_KERNEL_ATTN_MERGE, st, attn_merge_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st,
                               part, lse, p.splits, rows, static_cast<uint16_t *>(out));
        }
        return launch_status();
    }
    if (dtype == DDTREE_DTYPE_FP32)
        DDT_LAUNCH(DDTREE_KERNEL_ATTN_GENERIC, st, attn_generic_kernel<float>, dim3(Hq, T, batch), dim3(kGenThreads), 0, st,
                           static_cast<const float *>(q), static_cast<const float *>(k_cache),
                           static_cast<const float *>(v_cache), static_cast<const float *>(k_tree),
                           static_cast<const float *>(v_tree), ancestor_mask, args, T, Hq, Hkv, D,
                           softmax_scale, static_cast<float *>(out));
    else
        DDT_LAUNCH(DDTREE_KERNEL_ATTN_GENERIC, st, attn_generic_kernel<uint16_t>, dim3(Hq, T, batch), dim3(kGenThreads), 0, st,
                           static_cast<const uint16_t *>(q), static_cast<const uint16_t *>(k_cache),
                           static_cast<const uint16_t *>(v_cache), static_cast<const uint16_t *>(k_tree),
                           static_cast<const uint16_t *>(v_tree), ancestor_mask, args, T, Hq, Hkv, D,
                           softmax_scale, static_cast<uint16_t *>(out));
    return launch_status();
}

