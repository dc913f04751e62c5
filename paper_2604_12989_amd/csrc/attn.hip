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
// so one K/V tile serves G*T rows.  A workgroup (8 waves, two per SIMD) owns 256 consecutive
// rows (32 per wave) and a contiguous range of 64-key tiles (split-KV; partial results are merged by
// attn_merge_kernel).  Per tile:
//   S^T = K Q^T   v_mfma_f32_32x32x16_bf16, A = K tile from LDS (row = key), B = Q^T held in
//                 registers for the whole kernel.  In the accumulator layout a lane then owns
//                 one query row, so the softmax max and sum are register-local reductions.
//   P^T           exp2 of the scaled, masked scores; the accumulator registers of S^T are, as
//                 they stand, the B operand of the next product (no cross-lane movement).
//   O^T += V^T P^T  A = V^T, gathered from the row-major V tile in LDS by the transposing
//                 LDS read, in the key order the P^T registers happen to have.
// The softmax reference of a row is fixed by its first visible key, so the accumulators are
// never rescaled; a row whose scores outgrow its reference by more than 2^64 (rare) makes the
// workgroup redo its key range once with the true row maxima as references.
// K and V tiles sit in LDS as [key][dim]: K rows padded to 272 B, V rows of 256 B with their
// 64-byte blocks swizzled by the row, so that the 16-byte K reads and the transposing V reads are
// free of bank conflicts.
// The ancestor mask touches only the tree tiles (the last ceil(T/64) tiles): one 64-bit word per
// (row, tile), bit test per score.  Cache tiles carry no mask work at all.
#include <algorithm>
#include <vector>

#include "common.hpp"

namespace ddt {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;

// Eight waves of 32 query rows, two waves per SIMD with 256 registers each, so that one wave's
// waits (LDS, matrix results, barrier) are filled by the other; everything fits the 256
// architectural registers and no accumulation registers are used (asking for any would make the
// compiler split the budget 128 / 128 and spill).  Four waves of 64 rows with 512 registers each
// read half as much from LDS per matrix instruction but have nothing to fill a stall with
// (measured slower, in the kernel and in a micro-benchmark of the loop alone).
constexpr int kWaves = 8;
constexpr int kAttnThreads = 64 * kWaves;
constexpr int kKT = 64;        // keys per tile
constexpr int kHD = 128;       // head dim of the MFMA path
constexpr float kLog2e = 1.4426950408889634f;
constexpr int kAttnStages = 4;  // a power of two: the stage of tile i is i & 3
constexpr int kKRowBytes = 272;                  // K tile row in LDS: 256 B + 16 B pad (17 chunks)
constexpr int kVRowBytes = 256;                  // V tile row in LDS: no pad, 64-byte blocks swizzled by the row
constexpr int kKTileBytes = kKT * kKRowBytes;    // 17408 = 17 DMA blocks of 1 KB
constexpr int kVTileBytes = kKT * kVRowBytes;    // 16384 = 16 DMA blocks of 1 KB
constexpr int kStageBytes = kKTileBytes + kVTileBytes;
constexpr int kRingBytes = kAttnStages * kStageBytes;
// Behind the ring: the ancestor-mask words of the workgroup's rows for up to kMaskStages tree tiles
// of its key range, one 64-bit word per (tree tile, row), staged once by the prologue so that the
// masked steps read LDS and no global load sits in the key loop.
constexpr int kMaskStages = 8;
constexpr int kMaskStageBytes = kWaves * 32 * 8;
constexpr int kAttnLdsBytes = 256 + kRingBytes + kMaskStages * kMaskStageBytes;  // 256: the ring starts on a 256-byte boundary
static_assert(kAttnLdsBytes <= 160 * 1024, "fits the LDS of a compute unit");

struct AttnArgs {
    int32_t kv_start[DDTREE_MAX_BATCH];  // first cache row of each sequence
    int32_t kv_len[DDTREE_MAX_BATCH];    // its number of cache rows
    // matrix-core kernel only: the sequences longest cache first -- entry p = {sequence, its
    // first cache row, its number of cache rows, 0}, one 16-byte scalar load -- and the first work
    // item of each of the 8 XCDs' runs (run x = work items xcd_start[x] .. xcd_start[x + 1] - 1)
    int32_t by_length[DDTREE_MAX_BATCH][4];
    int32_t xcd_start[9];
    // Reciprocals for the divisions of the work-item decode, ceil(2^32 / d): x / d = mulhi(x, magic)
    // whenever x * d < 2^32.  0 where d = 1 or where the host could not guarantee that bound (the
    // kernel then divides).
    int32_t group_size;                  // G = Hq / Hkv
    uint32_t g_magic;                    // d = G, x = a row index
    uint32_t per_grp_magic;              // d = work items per (sequence, kv head), x = a work item
    uint32_t main_tiles_magic;           // d = whole row tiles, x = a work item within its group
    uint32_t hkv_magic;                  // d = Hkv, x = a group
    uint32_t splits_magic[2];            // d = key ranges of a whole / of the tail tile, x = key tiles * range + d - 1
};

__host__ __device__ __forceinline__ uint32_t magic_of(uint64_t d, uint64_t x_max)
{
    return (d >= 2 && x_max * d < 0x100000000ull) ? (uint32_t)((0x100000000ull + d - 1) / d) : 0u;
}
__host__ __device__ __forceinline__ int div_by(int x, int d, uint32_t magic)
{
    return magic != 0u ? (int)(((uint64_t)(uint32_t)x * magic) >> 32) : (d == 1 ? x : x / d);
}

// Shapes of the matrix-core kernel.  (The bound on the KV heads keeps the pitch between cache
// rows below 2^24 bytes, which the kernel's 24-bit address multiplies rely on.)
static bool mfma_shape(int dtype, int D, int Hkv) { return dtype == DDTREE_DTYPE_BF16 && D == kHD && Hkv <= 32768; }

AttnPlan attn_plan(int batch, int T, int Hq, int Hkv, int D, long long sum_L, int dtype)
{
    AttnPlan p{};
    p.splits = 1;
    if (!mfma_shape(dtype, D, Hkv)) return p;  // generic path needs no scratch
    const int G = Hq / Hkv;
    const long long M = (long long)T * G;
    const int nblk = (int)((M + 31) / 32);
    p.n_tiles = (nblk + 7) / 8;
    p.blk_base = nblk / p.n_tiles;
    p.blk_extra = nblk % p.n_tiles;
    const long long tiles = (sum_L / batch + T) / kKT;  // key tiles per sequence, roughly
    const long long base = (long long)batch * Hkv * p.n_tiles;  // workgroups per split
    // One workgroup per compute unit and launch round: base * S workgroups take
    // ceil(base * S / 256) rounds of 1/S of the key range each.  Take the S that minimises that
    // time, charged 2 % per split for the partials it writes and the merge reads, with at least
    // 4 key tiles per split.
    int best_s = 1;
    double best_cost = 1e30;
    for (int S = 1; S <= 32; ++S) {
        if (S > 1 && (long long)S * 4 > tiles) break;
        const long long rounds = (base * S + 255) / 256;
        const double cost = (double)rounds / S * (1.0 + 0.02 * (S - 1));
        if (cost < best_cost - 1e-12) {
            best_cost = cost;
            best_s = S;
        }
    }
    p.splits = best_s;
    p.part_splits = best_s;
    // Uneven form: when the blocks are a few more than whole tiles of 8 (T = 257 with four heads per
    // KV head: 33 blocks), even tiling leaves a fifth of the wave slots idle at no gain in time (a
    // tile is as slow as its busiest SIMD).  Whole tiles plus one small tail tile, the tail cut
    // into fewer key ranges because it runs about twice as fast per key tile, fills the 256 compute
    // units with shorter key ranges.  Taken when everything fits one round and the model says so.
    const int full = nblk / 8, rem = nblk % 8;
    if (full >= 1 && rem >= 1 && rem <= 4 && tiles >= 1) {
        const double c_tail = 0.6;  // a key tile of the small tail tile against one of a whole tile (measured)
        best_cost *= 0.97;  // (with key ranges the uneven form goes through partials: it has to pay for them)
        const long long base_m = (long long)batch * Hkv * full, base_t = (long long)batch * Hkv;
        for (int Sm = 1; Sm <= 32; ++Sm) {
            if (Sm > 1 && (long long)Sm * 4 > tiles) break;
            for (int St = 1; St <= 32; ++St) {
                if (St > 1 && (long long)St * 4 > tiles) break;
                if (base_m * Sm + base_t * St > 256) break;
                const double t_m = (double)((tiles + Sm - 1) / Sm), t_t = c_tail * (double)((tiles + St - 1) / St);
                const int smax = Sm > St ? Sm : St;
                const double cost = (t_m > t_t ? t_m : t_t) / (double)(tiles > 0 ? tiles : 1) * (1.0 + 0.02 * (smax - 1));
                if (cost < best_cost - 1e-12) {
                    best_cost = cost;
                    p.n_tiles = full + 1;
                    p.blk_base = 8;
                    p.blk_extra = rem;  // (read as: blocks of the tail tile)
                    p.splits = Sm;
                    p.tail_splits = St;
                    p.part_splits = smax;
                }
            }
        }
    }
    size_t off = 0;
    if (p.part_splits > 1) {
        const size_t rows = (size_t)batch * T * Hq;  // indexed by global row
        p.part_off = off;
        off = align_up(off + (size_t)p.part_splits * rows * D * 2, 256);  // fp16 partials
        p.lse_off = off;
        off = align_up(off + (size_t)p.part_splits * rows * 8, 256);      // (log2-sum-exp, scale) per row
    }
    p.bytes = off;
    return p;
}

// Upper bound of attn_plan(...).bytes over all sum_L.  In the even form the key ranges only shrink
// in number with shorter caches; in the uneven form the rounding of key tiles per range moves the
// optimum around, so the bound there is what one round of workgroups allows at all.
size_t attn_ws_upper(int batch, int T, int Hq, int Hkv, int D)
{
    AttnPlan p = attn_plan(batch, T, Hq, Hkv, D, (long long)1 << 40, DDTREE_DTYPE_BF16);
    int cap = p.part_splits;
    const int G = Hq / Hkv;
    const int nblk = (int)(((long long)T * G + 31) / 32);
    const int full = nblk / 8, rem = nblk % 8;
    const long long base_m = (long long)batch * Hkv * full, base_t = (long long)batch * Hkv;
    bool uneven_possible = false;
    if (full >= 1 && rem >= 1 && rem <= 4 && base_m + base_t <= 256) {
        uneven_possible = true;  // (it stores partials even with a single key range)
        long long sm = (256 - base_t) / base_m;
        if (sm > 32) sm = 32;
        if ((int)sm > cap) cap = (int)sm;
    }
    if (cap <= 1 && !uneven_possible) return p.bytes;
    const size_t rows = (size_t)batch * T * Hq;
    size_t off = align_up((size_t)cap * rows * D * 2, 256);
    off = align_up(off + (size_t)cap * rows * 8, 256);
    return off > p.bytes ? off : p.bytes;
}

__device__ __forceinline__ uint32_t pack_lo(uint32_t a, uint32_t b) { return (a & 0xFFFFu) | (b << 16); }
__device__ __forceinline__ uint32_t pack_hi(uint32_t a, uint32_t b) { return (a >> 16) | (b & 0xFFFF0000u); }
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
// two floats -> packed bf16 pair (round to nearest even), one v_cvt_pk_bf16_f32
__device__ __forceinline__ uint32_t f2bf_pair(float lo, float hi)
{
    const floatx2 f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}

// two floats -> packed fp16 pair (round to nearest even)
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t f2h_pair(float lo, float hi)
{
    const f16x2 h = {(_Float16)lo, (_Float16)hi};
    return __builtin_bit_cast(uint32_t, h);
}

// Compile-time loop: f(IC<B>{}), ..., f(IC<E-1>{}); the index is a constant expression inside f,
// as the immediate operands of the asm helpers below require.
template <int N>
struct IC {
    static constexpr int value = N;
};
template <int B, int E, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (B < E) {
        f(IC<B>{});
        static_for<B + 1, E>(f);
    }
}

// Reads of the K/V tiles are written as asm.  The tiles are filled by LDS-DMA
// (global_load_lds); the compiler cannot tell which stage a given LDS read touches and would
// wait for every outstanding tile load before each read, serialising prefetch and compute.  With
// asm reads the waits are placed by hand: s_waitcnt vmcnt(0) + barrier once per tile for the
// DMA, lds_wait_*() below for the reads (LDS reads return in order, so "at most N outstanding"
// identifies exactly which of them have landed).
// The destination of a read is tied to its previous value ("+v"): the read lands in the register
// of the operand it replaces and cannot be scheduled above the matrix instruction that still
// reads that operand.
template <int OFF>
__device__ __forceinline__ void lds_rd128(u32x4 &v, uint32_t addr)
{
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "+v"(v) : "v"(addr), "n"(OFF) : "memory");
}
// LDS transpose read (ds_read_b64_tr_b16).  Within each group of 16 lanes, lane 4*j + r points
// at four consecutive 16-bit elements; afterwards lane i of the group holds, for j = 0..3, element
// i % 4 of what lane 4*j + i / 4 pointed at.  With lane 4*j + r pointing at V[key_j][d0 + 4*r ..],
// lane i receives V[key_0..3][d0 + i]: a column of the row-major V tile, which is what the A
// operand (V^T) of the second product needs.
template <int OFF>
__device__ __forceinline__ void lds_rdtr(u32x2 &v, uint32_t addr)
{
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "+v"(v) : "v"(addr), "n"(OFF) : "memory");
}
// Wait for every outstanding LDS read of the wave; the operands tie the wait to the registers it
// protects so that their uses cannot be scheduled above it.
__device__ __forceinline__ void lds_wait_all(u32x4 (&k)[8], u32x2 (&v)[2][4][2])
{
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(k[0]), "+v"(k[1]), "+v"(k[2]), "+v"(k[3]), "+v"(k[4]), "+v"(k[5]), "+v"(k[6]), "+v"(k[7]),
                   "+v"(v[0][0][0]), "+v"(v[0][0][1]), "+v"(v[0][1][0]), "+v"(v[0][1][1]), "+v"(v[0][2][0]),
                   "+v"(v[0][2][1]), "+v"(v[0][3][0]), "+v"(v[0][3][1]), "+v"(v[1][0][0]), "+v"(v[1][0][1]),
                   "+v"(v[1][1][0]), "+v"(v[1][1][1]), "+v"(v[1][2][0]), "+v"(v[1][2][1]), "+v"(v[1][3][0]),
                   "+v"(v[1][3][1])
                 :
                 : "memory");
}

// Largest row sum (in units of 2^reference) a key range may end with: every single probability is
// then at most 2^72, far inside what bf16 operands and fp32 accumulators carry exactly as well as
// small ones.  A larger (or non-finite) sum means some score outgrew the row's reference by more
// than that and the workgroup redoes its key range with the true row maxima as references.
constexpr float kSumLimit = 0x1p72f;

template <int N>
__device__ __forceinline__ void vm_wait()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

__global__ __launch_bounds__(kAttnThreads) __attribute__((amdgpu_waves_per_eu(2, 2)))
void attn_mfma_kernel(const uint16_t *__restrict__ q, const uint16_t *__restrict__ k_cache,
                      const uint16_t *__restrict__ v_cache, const uint16_t *__restrict__ k_tree,
                      const uint16_t *__restrict__ v_tree, const uint64_t *__restrict__ mask,
                      AttnArgs args, int batch_n, int T, int Hq, int Hkv, float scale_log2e, int n_tiles_m,
                      int blk_base, int blk_extra, int main_splits, int tail_splits, int part_splits,
                      uint16_t *__restrict__ out,
                      uint16_t *__restrict__ part, float2 *__restrict__ lse)
{
    // LDS: kAttnStages stages of {K tile, V tile}, filled by direct global->LDS loads.  One wave
    // instruction writes 64 x 16 B contiguously, but every lane may fetch any 16-byte chunk, so
    // the layout within a tile is free.  K rows are padded to 17 chunks (272 B; the lanes that
    // land on padding fetch a dummy chunk): the 16-byte K reads are free of bank conflicts and
    // every read address is one per-lane base plus an immediate.  V rows are 256 B with their four
    // 64-byte blocks stored at position (block ^ (row & 3)): a transposing V read takes, in each
    // half-wave, two 32-byte pieces of one block from four consecutive rows, and the swizzle
    // spreads those over all 64 banks (rows padded to 288 B put the two pieces of row r and of
    // row r + 1 on the same 8 banks: 2 conflict cycles per read by the counters).  The block a
    // lane reads is (db ^ (row & 3)): an exclusive-or of the per-lane base with db * 64.
    extern __shared__ __align__(16) unsigned char smem_raw[];
    unsigned char *const smem =
        smem_raw + ((0u - (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem_raw) & 255u);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  The grid is read as
    // 8 runs of consecutive work items, run x being what XCD x executes, and consecutive
    // work items are the row tiles of one (group, key range): the row tiles that read the same K
    // and V rows share an L2, and those rows leave HBM once.  The host cuts the runs so that
    // each holds an eighth of the keys to visit (sequences of a ragged batch differ in length)
    // and lists the sequences longest first, so that an XCD's long work items start early.
    // The work items of a group are its main tiles, row tile fastest within a key range, then (in
    // the uneven form) the key ranges of its tail tile.
    const int main_tiles = tail_splits > 0 ? n_tiles_m - 1 : n_tiles_m;
    const int per_grp = main_tiles * main_splits + tail_splits;
    const int xcd = (int)blockIdx.x & 7;
    const int wid = args.xcd_start[xcd] + ((int)blockIdx.x >> 3);
    if (wid >= args.xcd_start[xcd + 1]) return;
    // (the divisions of this decode are multiplications by the host's reciprocals: a division by a
    // run-time value is some thirty instructions, and all of this sits before the first tile request)
    const int grp = div_by(wid, per_grp, args.per_grp_magic);  // (sequence, kv head) pair
    const int wg = wid - grp * per_grp;
    const bool tail = wg >= main_tiles * main_splits;
    const int wg_split = div_by(wg, main_tiles, args.main_tiles_magic);
    const int mt = tail ? main_tiles : wg - wg_split * main_tiles;
    const int split = tail ? wg - main_tiles * main_splits : wg_split;
    const int splits = tail ? tail_splits : main_splits;  // key ranges of this tile
    const int grp_seq = div_by(grp, Hkv, args.hkv_magic);
    const int hk = grp - grp_seq * Hkv;
    const int seq = args.by_length[grp_seq][0];
    const int G = args.group_size;
    const int W = (T + 63) >> 6;
    const int M = T * G;
    const int L0 = args.by_length[grp_seq][1];
    const int L = args.by_length[grp_seq][2];
    // this tile's blocks of 32 rows: wave w owns block w of the tile
    const int first_blk = tail_splits > 0 ? mt * 8 : mt * blk_base + min(mt, blk_extra);
    const int n_blk = tail_splits > 0 ? (tail ? blk_extra : 8) : blk_base + (mt < blk_extra ? 1 : 0);
    const int m0 = first_blk * 32;
    const int m_end = min(M, (first_blk + n_blk) * 32);
    const int last_node = min(T - 1, div_by(m_end - 1, G, args.g_magic));
    const int n_cache_tiles = (L + kKT - 1) / kKT;
    const int n_tree_tiles = last_node / kKT + 1;
    const int nt = n_cache_tiles + n_tree_tiles;
    // key ranges rounded up, so that a surplus tile goes to the early ranges: the last range holds
    // the tree tiles, which carry the mask work on top
    // (nt < 2^25 key tiles and at most 32 key ranges: 32-bit arithmetic is exact)
    const uint32_t s_magic = args.splits_magic[tail ? 1 : 0];
    const int t_begin = div_by(nt * split + splits - 1, splits, s_magic);
    const int t_end = div_by(nt * (split + 1) + splits - 1, splits, s_magic);
    const bool wave_active = m0 + wave * 32 < m_end;

    // Nothing derived from the lane's row is kept through the key loop: the masked steps, the
    // fetch of the row's own mask bit and the epilogue work the row out again from the thread
    // index (a handful of instructions), read through an empty statement so that the compiler does
    // not fall back on one copy -- held through the key loop, such values were spilled.
    auto lane_row = [&](int &rm, bool &rv, int &nd) __attribute__((always_inline)) {
        int t = (int)threadIdx.x;
        asm volatile("" : "+v"(t));
        rm = m0 + ((t >> 6) << 5) + (t & 31);
        rv = rm < m_end;
        nd = rv ? div_by(rm, G, args.g_magic) : 0;
    };
    auto mask_row = [&](int nd) __attribute__((always_inline)) { return mask + ((size_t)seq * T + nd) * W; };
    // the mask word that holds the row's own bit (a real tree node sees itself; padding rows produce
    // zeros) is requested during the last key tile and looked at in the epilogue: asked for here it
    // would hold a register through the whole loop, or be waited for and spilled before the loop
    uint32_t own_word = 0u;

    const uint32_t row_bytes = (uint32_t)Hkv * kHD * 2;  // bytes between consecutive keys in global memory
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    // first cache row and first tree row of this (sequence, kv head), as byte addresses; a tile is
    // kKT consecutive keys, tile_bytes apart (the cache bases are formed but never used when the
    // sequence has no cache rows)
    const unsigned char *const kc0 = reinterpret_cast<const unsigned char *>(k_cache) + ((size_t)L0 * Hkv + hk) * (kHD * 2);
    const unsigned char *const vc0 = reinterpret_cast<const unsigned char *>(v_cache) + ((size_t)L0 * Hkv + hk) * (kHD * 2);
    const unsigned char *const kt0 = reinterpret_cast<const unsigned char *>(k_tree) + ((size_t)seq * T * Hkv + hk) * (kHD * 2);
    const unsigned char *const vt0 = reinterpret_cast<const unsigned char *>(v_tree) + ((size_t)seq * T * Hkv + hk) * (kHD * 2);
    const uint32_t tile_bytes = (uint32_t)kKT * row_bytes;
    const int n_tiles = t_end - t_begin;
    // ---- tile loads: a K tile is 17 and a V tile 16 DMA blocks of 1 KB of LDS; lane l of block b fills
    //      16-byte slot u = 64*b + l, i.e. row u / chunks_per_row, chunk position u % chunks_per_row.
    //      The blocks are dealt round-robin to the n_dma loading waves: all eight, or, in a workgroup
    //      where at most two waves have query rows (the small tail tile), the six or seven waves
    //      without any, so that the waves that compute issue no loads at all.  A loading wave
    //      issues 2 K + 2 V blocks per tile plus at most one more of each: 4, 5 or 6 loads, the
    //      same for whole and ragged tiles (see tiles_in_flight).  The per-lane source offsets
    //      (bytes from the tile's first key) are computed once. ----
    const int n_active = min(kWaves, (m_end - m0 + 31) >> 5);  // waves 0 .. n_active-1 have query rows
    const bool offload = n_active <= 2;
    const int n_dma = offload ? kWaves - n_active : kWaves;
    const int dma_rank = offload ? wave_u - n_active : wave_u;  // negative: this wave loads nothing
    const bool k_third = dma_rank >= 0 && 2 * n_dma + dma_rank < 17;
    const bool v_third = dma_rank >= 0 && 2 * n_dma + dma_rank < 16;
    const int dma_loads = dma_rank < 0 ? 0 : 4 + (k_third ? 1 : 0) + (v_third ? 1 : 0);
    uint32_t k_src[3], v_src[3];   // of block n_dma*i + dma_rank
#pragma unroll
    for (int i = 0; i < 3; ++i) {
        const int u = (n_dma * i + max(dma_rank, 0)) * 64 + lane;
        const int rk = (u * 241) >> 12;   // u / 17 for u < 2048
        const int ck = u - rk * 17;
        // (24-bit multiplies: a row index below 64 times a row pitch below 2^24 -- the full multiply-add
        // leaves its result in a register pair, and six such pairs were kept through the kernel)
        k_src[i] = __umul24((uint32_t)min(rk, kKT - 1), row_bytes) + (ck == 16 ? 0 : ck) * 16;  // padding slot: any chunk
        const int rv = u >> 4, cv = (u & 15) ^ ((rv & 3) << 2);  // slot (row, position) holds chunk position ^ 4 (row & 3)
        v_src[i] = __umul24((uint32_t)min(rv, kKT - 1), row_bytes) + cv * 16;
    }
    auto issue_tile = [&](int tt, int stage) __attribute__((always_inline)) {
        const bool cache = tt < n_cache_tiles;
        const int tl = cache ? tt : tt - n_cache_tiles;
        const uint64_t toff = (uint64_t)(uint32_t)tl * tile_bytes;
        const unsigned char *kp = (cache ? kc0 : kt0) + toff;
        const unsigned char *vp = (cache ? vc0 : vt0) + toff;
        const int valid_ = min(kKT, (cache ? L : T) - tl * kKT);
        unsigned char *st = smem + stage * kStageBytes;
        // Every load is written as (uniform 64-bit base) + (32-bit lane offset), the form that
        // takes the base in scalar registers; the offsets pass through an empty asm so that their
        // widening to 64 bits stays next to the load instead of being kept, widened, in a pair of
        // vector registers each for the whole kernel.
        auto dma = [&](const unsigned char *base, uint32_t off, unsigned char *dst) __attribute__((always_inline)) {
            asm volatile("" : "+v"(off));
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(base + off),
                                             (__attribute__((address_space(3))) void *)dst, 16, 0, 0);
        };
        if (dma_rank < 0) return;
        if (valid_ == kKT) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                dma(kp, k_src[i], st + (n_dma * i + dma_rank) * 1024);
                dma(vp, v_src[i], st + kKTileBytes + (n_dma * i + dma_rank) * 1024);
            }
            if (k_third) dma(kp, k_src[2], st + (2 * n_dma + dma_rank) * 1024);
            if (v_third) dma(vp, v_src[2], st + kKTileBytes + (2 * n_dma + dma_rank) * 1024);
        } else {
            // ragged tile (at most two per key range): rows past the end re-read the last valid
            // row, so that the LDS tile holds finite data everywhere
#pragma unroll 1
            for (int i = 0; i < 3; ++i) {
                const int blk = n_dma * i + dma_rank;
                const int u = blk * 64 + lane;
                if (blk < 17) {
                    const int r = (u * 241) >> 12, c = u - r * 17;
                    dma(kp, __umul24((uint32_t)min(r, valid_ - 1), row_bytes) + (c == 16 ? 0 : c) * 16, st + blk * 1024);
                }
                if (blk < 16) {
                    const int r = u >> 4, c = (u & 15) ^ ((r & 3) << 2);
                    dma(vp, __umul24((uint32_t)min(r, valid_ - 1), row_bytes) + c * 16, st + kKTileBytes + blk * 1024);
                }
            }
        }
    };
    // Wait until at most the `n` most recently requested tiles of this wave may still be in
    // flight (vector memory operations complete in order, and a tile is dma_loads of them for
    // this wave): everything requested before them has landed.
    auto tiles_in_flight = [&](int n) __attribute__((always_inline)) {
        if (n <= 0 || dma_loads == 0) vm_wait<0>();
        else if (dma_loads == 6) { if (n == 1) vm_wait<6>(); else vm_wait<12>(); }
        else if (dma_loads == 5) { if (n == 1) vm_wait<5>(); else vm_wait<10>(); }
        else { if (n == 1) vm_wait<4>(); else vm_wait<8>(); }
    };

    // Everything in LDS is addressed from a 256-byte boundary: the V operand addresses below take
    // an exclusive-or on bits 6 and 7.
    const uint32_t lds_base = ((uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem_raw + 255u) & ~255u;

    // ---- the first requests: the first key tile, the queries and mask words, two more key tiles.
    //      Vector memory operations complete in order, so the wait for "all but the last tile
    //      requested" further down also covers the queries and the mask words. ----
    if (n_tiles > 0) issue_tile(t_begin, 0);
    __builtin_amdgcn_sched_barrier(0);
    // Q^T operand: lane holds Q[row][16*ks + 8*half .. +8]
    bf16x8 qreg[8];
    // ancestor-mask words of this lane's row for the first kMaskStages tree tiles of the key range
    const int tb0 = max(t_begin - n_cache_tiles, 0);                       // first tree tile of the range
    const int n_stage = max(0, min(t_end - n_cache_tiles - tb0, kMaskStages));  // how many are staged in LDS
    uint64_t mword[kMaskStages];
    {
        int rm, nd;
        bool rv;
        lane_row(rm, rv, nd);
        const size_t rowg = (size_t)(seq * T + nd) * Hq + hk * G + (rv ? rm - nd * G : 0);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (rv) v = *reinterpret_cast<const uint4 *>(q + rowg * kHD + ks * 16 + half * 8);
            qreg[ks] = __builtin_bit_cast(bf16x8, v);
        }
#pragma unroll
        for (int i = 0; i < kMaskStages; ++i) mword[i] = (rv && i < n_stage) ? mask_row(nd)[tb0 + i] : 0ull;
    }
    __builtin_amdgcn_sched_barrier(0);
    if (n_tiles > 1) issue_tile(t_begin + 1, 1);
    if (n_tiles > 2) issue_tile(t_begin + 2, 2);
    __builtin_amdgcn_sched_barrier(0);
    // LDS address of this lane's row in the staged mask words (both half-waves of a row read the
    // same word); tree tile tb0 + i is kMaskStageBytes * i further on
    auto mask_lds = [&]() __attribute__((always_inline)) {
        int t = (int)threadIdx.x;
        asm volatile("" : "+v"(t));
        return lds_base + (uint32_t)(kRingBytes + ((t >> 6) << 8) + ((t & 31) << 3));
    };

    // per-lane LDS read bases (bytes, relative to the tile); everything else is an immediate
    const int k_base = l32 * kKRowBytes + half * 16;  // K: row l32 (+32*kb), column 2*ks + half
    const int lm = lane & 15, dim16 = (lane >> 4) & 1;
    // V: row 4*half + lm/4 (+16*kstep, +8), dims 32*db + 16*dim16 + 4*(lm%4); the 64-byte block db of
    // a row sits at position db ^ (row & 3), and row & 3 = lm / 4 for every row this lane reads: the
    // base points at block (row & 3), the position of db = 0, and a read takes base ^ (db * 64)
    const int v_base = kKTileBytes + (4 * half + (lm >> 2)) * kVRowBytes + ((lm >> 2) << 6) + 32 * dim16 + 8 * (lm & 3);
    static_assert((kKTileBytes & 0xFF) == 0 && (kStageBytes & 0xFF) == 0 && (kVRowBytes & 0xFF) == 0,
                  "bits 6 and 7 of a V operand address come from the block position alone");

    // Operand staging registers: K rows of one 32-key sub-tile (8 k-steps over the head dim) and
    // V columns of one sub-tile (2 k-steps x 4 dim blocks x 2 transposing reads).
    u32x4 kbuf[8];
    u32x2 vbuf[2][4][2];
#pragma unroll
    for (int i = 0; i < 8; ++i) kbuf[i] = (u32x4){0u, 0u, 0u, 0u};
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) vbuf[a][b][0] = vbuf[a][b][1] = (u32x2){0u, 0u};
    floatx16 o[4];      // O^T accumulators, one per block of 32 output dims
    floatx16 s_a, s_b;  // scores of two consecutive sub-tiles (one being turned into P, one being formed)
    uint32_t p_a[8], p_b[8];  // P^T operands of two consecutive sub-tiles, bf16 pairs
    float m_ref = -INFINITY;   // softmax reference of the row (log2 units): fixed by its first visible keys
    float m_seen = -INFINITY;  // true running maximum, tracked only by the first pass of a retry
    // Row sums of P, taken by the matrix cores from the very bf16 values that multiply V: one
    // v_mfma_f32_16x16x32_bf16 per k-step whose B operand is the P^T operand as it stands and whose
    // A operand selects, for output row 0, the lanes that hold query rows 0-15 (lanes 0-15 and 32-47
    // of the P^T registers: k-groups 0 and 2 of the smaller shape) and, for output row 1, those that
    // hold query rows 16-31 (k-groups 1 and 3).  Lane j < 16 then holds the sum of query row j in
    // register 0 and that of row 16 + j in register 1.
    floatx4 l_acc = {0.0f, 0.0f, 0.0f, 0.0f};
    const uint32_t sel_bits = (lane == 0 || lane == 32 || lane == 17 || lane == 49) ? 0x3f803f80u : 0u;
    const bf16x8 sel = __builtin_bit_cast(bf16x8, (u32x4){sel_bits, sel_bits, sel_bits, sel_bits});
    auto row_sum = [&]() __attribute__((always_inline)) {
        const float lo = __shfl(l_acc[0], l32 & 15, 64), hi = __shfl(l_acc[1], l32 & 15, 64);
        return l32 < 16 ? lo : hi;
    };

    // One step of the software pipeline, sub-tile j (32 keys) of tile t:
    //   matrix cores   S(j+1) = K Q^T  (8 instructions)  and  O += V^T P(j-1)  (8 instructions), alternating
    //   vector ALUs    P(j) = 2^(S(j) * scale - reference), its row sum, bf16 pairs
    //   LDS            operands K(j+2) and V(j), each requested right behind the matrix instruction
    //                  that consumed the register it lands in
    // so that every matrix instruction has its share of the softmax (fma, exp, add, half a
    // conversion) issued in its shadow.  Slow steps (tiles with masked keys, the first tile of a key
    // range, retries) first apply the mask and fix the reference of rows that see their first key.
    auto step = [&](bool slow, floatx16 &cur, floatx16 &nxt, uint32_t (&pin)[8], uint32_t (&pout)[8],
                    uint32_t k_addr, uint32_t v_addr, int t, int kb, bool track, auto &&early) __attribute__((always_inline)) {
        lds_wait_all(kbuf, vbuf);
        bool dark = false;  // (uniform) no row of this wave sees any key of the sub-tile
        if (slow) {
            const bool is_tree = t >= n_cache_tiles;
            const int tb = t - n_cache_tiles;
            const int valid = is_tree ? min(kKT, T - tb * kKT) : min(kKT, L - t * kKT);
            uint32_t w32 = ~0u;
            if (is_tree || valid < kKT) {  // tree tiles and a ragged last cache tile
                uint64_t word = ~0ull;
                if (is_tree) {
                    if (tb - tb0 < n_stage) {
                        // staged by the prologue (zero for rows past the end); the wave has no
                        // other LDS read in flight at this point
                        u32x2 w2;
                        asm volatile("ds_read_b64 %0, %1\n\ts_waitcnt lgkmcnt(0)"
                                     : "=v"(w2)
                                     : "v"(mask_lds() + (uint32_t)((tb - tb0) * kMaskStageBytes))
                                     : "memory");
                        word = ((uint64_t)w2.y << 32) | w2.x;
                    } else {
                        int rm, nd;
                        bool rv;
                        lane_row(rm, rv, nd);
                        word = rv ? mask_row(nd)[tb] : 0ull;
                    }
                }
                if (valid < kKT) word &= (1ull << valid) - 1ull;
                // this lane's keys of the sub-tile: 8 * (v / 4) + 4 * half + v % 4
                w32 = ((uint32_t)(word >> (32 * kb)) >> (4 * half)) & 0x0F0F0F0Fu;
                // (a tree row sees its few ancestors and itself: most (row block, sub-tile) pairs of the
                // tree tiles are dark, and a dark sub-tile has no maximum to look at)
                dark = __builtin_amdgcn_ballot_w64(w32 != 0u) == 0ull;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    // all ones where the key is visible: the score stays, else it becomes -inf (two
                    // instructions per score, and no score of a hidden key, whatever its bits, survives)
                    const uint32_t keep = (uint32_t)__builtin_amdgcn_sbfe((int)w32, (v >> 2) * 8 + (v & 3), 1);
                    cur[v] = __uint_as_float((__float_as_uint(cur[v]) & keep) | (0xFF800000u & ~keep));
                }
            }
            // the maximum of the sub-tile is of interest only to rows still without a reference
            // (and to the pass that tracks the true maxima)
            if (!dark && (track || __builtin_amdgcn_ballot_w64(m_ref == -INFINITY) != 0ull)) {
                float tmax = cur[0];
#pragma unroll
                for (int v = 1; v < 16; ++v) tmax = fmaxf(tmax, cur[v]);
                // the other half-wave holds the other 16 keys of this row
                const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(tmax), __float_as_uint(tmax),
                                                                 false, false);
                tmax = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1])) * scale_log2e;
                if (track) m_seen = fmaxf(m_seen, tmax);
                m_ref = m_ref == -INFINITY ? tmax : m_ref;
            }
        }
        // The reference is never moved, so the accumulators are never rescaled: exp2 arguments may
        // become positive, which fp32 and bf16 carry exactly as well as negative ones.
        const float m_use = m_ref == -INFINITY ? 0.0f : m_ref;
        static_for<0, 8>([&](auto I) {
            constexpr int i = decltype(I)::value;
            {
                const bf16x8 a = __builtin_bit_cast(bf16x8, kbuf[i]);
                if constexpr (i == 0) {
                    floatx16 z;
#pragma unroll
                    for (int v = 0; v < 16; ++v) z[v] = 0.0f;
                    nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[i], z, 0, 0, 0);
                } else {
                    nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[i], nxt, 0, 0, 0);
                }
                lds_rd128<i * 32>(kbuf[i], k_addr);
            }
            float e0 = __builtin_amdgcn_exp2f(fmaf(cur[2 * i], scale_log2e, -m_use));
            // (the empty asm statements pin the softmax arithmetic to its slot: without them the
            // optimiser sinks it past the slot boundaries towards its first use in the next step)
            asm volatile("" : "+v"(e0));
            __builtin_amdgcn_sched_barrier(0);
            {
                // element j of the P^T operand of k-step t2 is key 16*t2 + 8*(j/4) + 4*half + j%4 of the
                // sub-tile; the two transposing reads fetched those keys
                constexpr int t2 = i / 4, db = i % 4;
                const bf16x8 a = __builtin_bit_cast(
                    bf16x8, (u32x4){vbuf[t2][db][0].x, vbuf[t2][db][0].y, vbuf[t2][db][1].x, vbuf[t2][db][1].y});
                const bf16x8 b = __builtin_bit_cast(
                    bf16x8, (u32x4){pin[4 * t2], pin[4 * t2 + 1], pin[4 * t2 + 2], pin[4 * t2 + 3]});
                o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, o[db], 0, 0, 0);
                if constexpr (db == 3) l_acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(sel, b, l_acc, 0, 0, 0);
                lds_rdtr<t2 * 16 * kVRowBytes>(vbuf[t2][db][0], v_addr ^ (uint32_t)(db * 64));
                lds_rdtr<(t2 * 16 + 8) * kVRowBytes>(vbuf[t2][db][1], v_addr ^ (uint32_t)(db * 64));
            }
            const float e1 = __builtin_amdgcn_exp2f(fmaf(cur[2 * i + 1], scale_log2e, -m_use));
            pout[i] = f2bf_pair(e0, e1);
            asm volatile("" : "+v"(pout[i]));
            __builtin_amdgcn_sched_barrier(0);
            // work that only has to happen some time during the step (the next tile request: scalar
            // address arithmetic and a handful of loads) goes behind the first slots, where the
            // other wave of the SIMD keeps the matrix cores busy meanwhile
            if constexpr (i == 1) {
                early();
                __builtin_amdgcn_sched_barrier(0);
            }
        });
    };

    // The mask words go to LDS once they are there (the wave has nothing else to do meanwhile: the
    // first key tile was requested before them).  A word is read back only by the lane that wrote
    // it and by its twin in the other half of the same wave.
    if (n_stage > 0 && half == 0) {
        const uint32_t a = mask_lds();
#pragma unroll
        for (int i = 0; i < kMaskStages; ++i)
            if (i < n_stage)
                asm volatile("ds_write_b64 %0, %1 offset:%2" ::"v"(a), "v"(mword[i]), "n"(i * kMaskStageBytes) : "memory");
    }

    // ---- the key range, up to three times: once normally; if some row's sum shows that its
    //      scores outgrew the reference, once more to find the true row maxima and a last time with
    //      those as references (rare) ----
    for (int pass = 0;; ++pass) {
        const bool all_slow = pass > 0, track = pass == 1;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[db][v] = 0.0f;
#pragma unroll
        for (int i = 0; i < 8; ++i) p_b[i] = 0u;
        l_acc = (floatx4){0.0f, 0.0f, 0.0f, 0.0f};
        // Ring of four stages: while the keys of tile `it` are worked on, tile it+1 is resident
        // (its K operands are requested one sub-tile ahead), tile it+2 is in flight and tile it+3
        // is requested into the stage that tile it-1 has just left.
        if (pass > 0) {  // (the first pass's tiles were requested at the top of the kernel)
            if (n_tiles > 0) issue_tile(t_begin, 0);
            if (n_tiles > 1) issue_tile(t_begin + 1, 1);
            if (n_tiles > 2) issue_tile(t_begin + 2, 2);
        }
        tiles_in_flight(n_tiles > 2 ? 1 : 0);  // tiles 0 and 1 have landed
        __syncthreads();
        if (wave_active && n_tiles > 0) {
            // S(0) on its own, then the operands the first step expects: K(1), and V(0) standing in
            // for the V(-1) that does not exist (P(-1) is zero)
            static_for<0, 8>([&](auto I) { lds_rd128<decltype(I)::value * 32>(kbuf[decltype(I)::value], lds_base + k_base); });
            lds_wait_all(kbuf, vbuf);
            static_for<0, 8>([&](auto I) {
                constexpr int i = decltype(I)::value;
                const bf16x8 a = __builtin_bit_cast(bf16x8, kbuf[i]);
                if constexpr (i == 0) {
                    floatx16 z;
#pragma unroll
                    for (int v = 0; v < 16; ++v) z[v] = 0.0f;
                    s_a = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[i], z, 0, 0, 0);
                } else {
                    s_a = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[i], s_a, 0, 0, 0);
                }
                lds_rd128<i * 32>(kbuf[i], lds_base + k_base + 32 * kKRowBytes);
            });
            static_for<0, 8>([&](auto I) {
                constexpr int t2 = decltype(I)::value / 4, db = decltype(I)::value % 4;
                lds_rdtr<t2 * 16 * kVRowBytes>(vbuf[t2][db][0], (lds_base + v_base) ^ (uint32_t)(db * 64));
                lds_rdtr<(t2 * 16 + 8) * kVRowBytes>(vbuf[t2][db][1], (lds_base + v_base) ^ (uint32_t)(db * 64));
            });
        }
        for (int it = 0; it < n_tiles; ++it) {
            const int t = t_begin + it;
            const uint32_t stage_addr = lds_base + (it & (kAttnStages - 1)) * kStageBytes;
            // when there is no next tile the K operands are re-read from this one and never used:
            // the control flow stays the same for the last tile
            const uint32_t next_addr = it + 1 < n_tiles ? lds_base + ((it + 1) & (kAttnStages - 1)) * kStageBytes : stage_addr;
            if (it > 0) {
                // Tile it+1 has landed (this wave's share; the barrier makes it everyone's) and
                // nobody reads tile it-1 any more: its stage takes tile it+3.
                if (wave_active) lds_wait_all(kbuf, vbuf);
                tiles_in_flight(it + 2 < n_tiles ? 1 : 0);
                __syncthreads();
            }
            auto request = [&]() __attribute__((always_inline)) {
                if (it + 3 < n_tiles) issue_tile(t + 3, (it + 3) & (kAttnStages - 1));
            };
            if (!wave_active) request();
            if (wave_active) {
                if (it == n_tiles - 1) {
                    int rm, nd;
                    bool rv;
                    lane_row(rm, rv, nd);
                    if (rv) own_word = reinterpret_cast<const uint32_t *>(mask_row(nd))[nd >> 5];
                }
                const bool slow = all_slow || it == 0 || t >= n_cache_tiles || (t == n_cache_tiles - 1 && (L & (kKT - 1)) != 0);
                // sub-tile (t, 0): forms S(t, 1), multiplies P(t-1, 1); requests K(t+1, 0) and V(t, 0)
                // sub-tile (t, 1): forms S(t+1, 0), multiplies P(t, 0); requests K(t+1, 1) and V(t, 1)
                step(slow, s_a, s_b, p_b, p_a, next_addr + k_base, stage_addr + v_base, t, 0, track, request);
                step(slow, s_b, s_a, p_a, p_b, next_addr + k_base + 32 * kKRowBytes,
                     stage_addr + v_base + 32 * kVRowBytes, t, 1, track, []() {});
            }
        }
        if (wave_active && n_tiles > 0) {
            // drain: P V of the last sub-tile
            lds_wait_all(kbuf, vbuf);
#pragma unroll
            for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
                for (int db = 0; db < 4; ++db) {
                    const bf16x8 a = __builtin_bit_cast(
                        bf16x8, (u32x4){vbuf[t2][db][0].x, vbuf[t2][db][0].y, vbuf[t2][db][1].x, vbuf[t2][db][1].y});
                    const bf16x8 b = __builtin_bit_cast(
                        bf16x8, (u32x4){p_b[4 * t2], p_b[4 * t2 + 1], p_b[4 * t2 + 2], p_b[4 * t2 + 3]});
                    o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, o[db], 0, 0, 0);
                    if (db == 3) l_acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(sel, b, l_acc, 0, 0, 0);
                }
        }
        // no DMA and no LDS read of this wave is still in flight; behind the barrier that holds for
        // the workgroup, and the ring may be filled again (or reused by the epilogue)
        __builtin_amdgcn_s_waitcnt(0);
        if (pass == 0) {
            const float l_tot = row_sum();
            const bool outgrown = wave_active && !(l_tot <= kSumLimit);  // also true for inf and NaN
            if (!__syncthreads_or(outgrown ? 1 : 0)) break;
            m_ref = -INFINITY;
            m_seen = -INFINITY;
        } else {
            __syncthreads();
            if (pass == 2) break;
            m_ref = m_seen;  // the true row maxima: nothing can outgrow them
        }
    }

    if (!wave_active) return;
    // ---- epilogue ----
    // A lane holds, of its row, sixteen groups of four output elements 8 bytes wide: stored from
    // there a row would leave in 32 pieces.  The block is staged row-major in this wave's share
    // of the ring (idle now: every wave has passed the barrier above with its tiles consumed, and
    // no DMA is in flight) and leaves in whole rows, 16 bytes per lane and four rows per store.
    constexpr int kEpiRow = kHD * 2 + 16;  // bytes per staged row: 16-byte aligned, rows 4 banks apart
    static_assert(kWaves * 32 * kEpiRow <= kAttnLdsBytes, "staging fits the ring");
    // (lane-derived addresses are formed here, from the thread index read afresh: formed from the
    // values at the top of the kernel they would be computed there and spilled)
    int e_tid = (int)threadIdx.x;
    asm volatile("" : "+v"(e_tid));
    const int e_lane = e_tid & 63, e_l32 = e_tid & 31, e_half = (e_tid >> 5) & 1, e_wave = e_tid >> 6;
    unsigned char *stg = smem + e_wave * (32 * kEpiRow);
    const size_t n_rows = (size_t)batch_n * T * Hq;
    {
        int e_row, e_node;
        bool e_valid;
        lane_row(e_row, e_valid, e_node);
        const float l_tot = row_sum();
        const bool real_ = (own_word >> (e_node & 31)) & 1u;
        const float inv = (e_valid && real_ && l_tot > 0.0f) ? 1.0f / l_tot : 0.0f;
        // The partial of a key range is stored as fp16 relative to the largest magnitude of its
        // row (so that it fits whatever the values are: bf16 inputs reach 3e38, fp16 65504), with
        // that magnitude kept beside the log2-sum-exp.
        float rs = 1.0f;
        if (part_splits != 0) {
            float amax = 0.0f;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) amax = fmaxf(amax, fabsf(o[db][v]));
            amax = fmaxf(amax, __shfl_xor(amax, 32, 64)) * inv;  // the other half-wave holds the row's other dims
            rs = (amax > 0.0f && amax < INFINITY) ? amax : 1.0f;
        }
        const float mul = part_splits == 0 ? inv : inv / rs;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const int dim = db * 32 + g4 * 8 + e_half * 4;
                const float a0 = o[db][4 * g4 + 0] * mul, a1 = o[db][4 * g4 + 1] * mul;
                const float a2 = o[db][4 * g4 + 2] * mul, a3 = o[db][4 * g4 + 3] * mul;
                uint2 val;  // bf16 for the output itself, fp16 for the partial of a key range
                val.x = part_splits == 0 ? f2bf_pair(a0, a1) : f2h_pair(a0, a1);
                val.y = part_splits == 0 ? f2bf_pair(a2, a3) : f2h_pair(a2, a3);
                *reinterpret_cast<uint2 *>(stg + e_l32 * kEpiRow + dim * 2) = val;
            }
        if (part_splits != 0 && e_valid && e_half == 0) {
            // log2-sum-exp and scale of this key range, indexed by global row
            const size_t ridx = (size_t)((seq * T + e_node) * Hq + hk * G + (e_row - e_node * G));
            lse[(size_t)split * n_rows + ridx] =
                make_float2(inv > 0.0f ? m_ref + __builtin_amdgcn_logf(l_tot) : -INFINITY, rs);
            // key ranges this tile does not have (the other kind of tile has more): empty
            if (split == 0)
                for (int sx = splits; sx < part_splits; ++sx) lse[(size_t)sx * n_rows + ridx] = make_float2(-INFINITY, 1.0f);
        }
    }
    uint16_t *dst_base = part_splits == 0 ? out : part + (size_t)split * n_rows * kHD;
    const int chunk = e_lane & 15;
    int r = m0 + e_wave * 32 + (e_lane >> 4);  // rows lane >> 4, + 4, + 8, ... of the block
    int node = div_by(r, G, args.g_magic), g = r - node * G;
#pragma unroll
    for (int rr = 0; rr < 8; ++rr) {
        if (r < m_end) {
            const uint4 v = *reinterpret_cast<const uint4 *>(stg + (rr * 4 + (e_lane >> 4)) * kEpiRow + chunk * 16);
            const size_t rg = (size_t)(seq * T + node) * Hq + hk * G + g;
            *reinterpret_cast<uint4 *>(dst_base + rg * kHD + chunk * 8) = v;
        }
        r += 4;
        g += 4;
        while (g >= G) {
            g -= G;
            ++node;
        }
    }
}

// Merge of the split-KV partials: out = sum_s 2^(lse_s - max) O_s / sum_s 2^(lse_s - max).
// Partials are normalised per split and stored as fp16 relative to the largest magnitude of the
// row, which travels beside the row's log2-sum-exp (eps 2^-11 is below the bf16 rounding of the
// result).  One thread per (row, 8 dims); the loads of kMergeBatch splits are in flight
// together: 8 for up to 8 key ranges, 16 beyond (small budgets on long caches).
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

template <int kMergeBatch>
__global__ __launch_bounds__(256) void attn_merge_kernel(const uint16_t *__restrict__ part_all,
                                                         const float2 *__restrict__ lse_all, size_t n_rows,
                                                         int splits, uint16_t *__restrict__ out)
{
    const size_t gid = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t row = gid >> 4;
    const int dg = (int)(gid & 15);
    if (row >= n_rows) return;
    const uint16_t *part = part_all + row * kHD + dg * 8;
    const float2 *lse = lse_all + row;
    const size_t pstride = n_rows * kHD;

    // one pass: the weights are taken against the largest lse seen so far and what has been
    // summed is rescaled when a batch brings a larger one
    float mx = -INFINITY;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    float wsum = 0.0f;
    for (int s0 = 0; s0 < splits; s0 += kMergeBatch) {
        f16x8 v[kMergeBatch];
        float l[kMergeBatch], sc[kMergeBatch];
#pragma unroll
        for (int j = 0; j < kMergeBatch; ++j) {
            const bool on = s0 + j < splits;
            const float2 ls = on ? lse[(size_t)(s0 + j) * n_rows] : make_float2(-INFINITY, 1.0f);
            l[j] = ls.x;
            sc[j] = ls.y;
            v[j] = on ? *reinterpret_cast<const f16x8 *>(part + (size_t)(s0 + j) * pstride) : f16x8(0);
        }
        float bm = l[0];
#pragma unroll
        for (int j = 1; j < kMergeBatch; ++j) bm = fmaxf(bm, l[j]);
        if (bm > mx) {
            const float r = mx > -INFINITY ? __builtin_amdgcn_exp2f(mx - bm) : 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] *= r;
            wsum *= r;
            mx = bm;
        }
#pragma unroll
        for (int j = 0; j < kMergeBatch; ++j) {
            // an empty key range (lse = -inf) has no partial behind it: whatever bits were
            // read there must not reach the sum, not even times zero
            const bool live = l[j] > -INFINITY;
            const float w = live ? __builtin_amdgcn_exp2f(l[j] - mx) : 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] += live ? (w * sc[j]) * (float)v[j][e] : 0.0f;
            wsum += w;
        }
    }
    const float inv = wsum > 0.0f ? 1.0f / wsum : 0.0f;
    uint4 val;
    val.x = f2bf_pair(acc[0] * inv, acc[1] * inv);
    val.y = f2bf_pair(acc[2] * inv, acc[3] * inv);
    val.z = f2bf_pair(acc[4] * inv, acc[5] * inv);
    val.w = f2bf_pair(acc[6] * inv, acc[7] * inv);
    *reinterpret_cast<uint4 *>(out + row * kHD + dg * 8) = val;
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
// eight consecutive elements (32- or 16-byte aligned: rows are multiples of eight elements long)
__device__ __forceinline__ void ld_elem8(const float *p, float (&o)[8])
{
    const float4 a = reinterpret_cast<const float4 *>(p)[0], b = reinterpret_cast<const float4 *>(p)[1];
    o[0] = a.x, o[1] = a.y, o[2] = a.z, o[3] = a.w, o[4] = b.x, o[5] = b.y, o[6] = b.z, o[7] = b.w;
}
__device__ __forceinline__ void ld_elem8(const uint16_t *p, float (&o)[8])
{
    const uint4 a = *reinterpret_cast<const uint4 *>(p);
    const uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        o[2 * i] = __uint_as_float(w[i] << 16);
        o[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
    }
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
    const int L0 = args.kv_start[seq];
    const int L = args.kv_len[seq];
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
    const int groups = kGenThreads / D;  // key groups of the P V product (D <= 256)
    const int gd = tid % D, gg = tid / D;
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
            // the key row in 16 elements per step (D is a multiple of 8), summed in element order
            int c = 0;
            for (; c + 16 <= D; c += 16) {
                float k0[8], k1[8];
                ld_elem8(krow + c, k0);
                ld_elem8(krow + c + 8, k1);
#pragma unroll
                for (int u = 0; u < 8; ++u) dot = fmaf(s_q[c + u], k0[u], dot);
#pragma unroll
                for (int u = 0; u < 8; ++u) dot = fmaf(s_q[c + 8 + u], k1[u], dot);
            }
            if (c < D) {
                float k0[8];
                ld_elem8(krow + c, k0);
#pragma unroll
                for (int u = 0; u < 8; ++u) dot = fmaf(s_q[c + u], k0[u], dot);
            }
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
        if (gg < groups) {
            // thread (gd, gg) accumulates output element gd over the keys gg, gg + groups, ...
            // of the tile, sixteen value rows in flight at a time; a masked key has weight 0 and
            // its row (a real tree row) is read all the same, so that no load waits for a branch
            acc *= alpha;
            const int cnt = min(kGenThreads, total - j0);
            auto vrow = [&](int jj) -> const TIO * {
                return jj < L ? v_cache + ((size_t)(L0 + jj) * Hkv + hk) * D
                              : v_tree + (((size_t)seq * T + (jj - L)) * Hkv + hk) * D;
            };
            int t = gg;
            for (; t + 15 * groups < cnt; t += 16 * groups) {
                float vv[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) vv[u] = ld_elem(vrow(j0 + t + u * groups) + gd);
#pragma unroll
                for (int u = 0; u < 16; ++u) acc = fmaf(s_p[t + u * groups], vv[u], acc);
            }
            for (; t < cnt; t += groups) acc = fmaf(s_p[t], ld_elem(vrow(j0 + t) + gd), acc);
        }
        __syncthreads();
    }
    // the key groups' partial sums of each output element
    s_p[tid] = gg < groups ? acc : 0.0f;
    __syncthreads();
    if (tid < D) {
        float o = 0.0f;
        for (int g = 0; g < groups; ++g) o += s_p[g * D + tid];
        st_elem(orow + tid, l_run > 0.0f ? o / l_run : 0.0f);
    }
}

}  // namespace ddt

// The launch tables of the matrix-core kernel for a plan: reciprocals for the work-item decode, the
// sequences by length, the cut of the work items into the 8 XCDs' runs.  *grid_x = workgroups to
// launch.  False if the launch would exceed 2^28 work items.
static bool attn_fill_args(ddt::AttnArgs &args, const ddt::AttnPlan &p, const int32_t *kv_start,
                           const int32_t *kv_len, int batch, int T, int Hkv, long long *grid_x)
{
    using namespace ddt;
    const int main_tiles = p.tail_splits > 0 ? p.n_tiles - 1 : p.n_tiles;
    // Work items in launch order: sequences longest first, then kv head, then the items of
    // the group.  An item visits about (L + T) / splits keys; the 8 runs are cut where the
    // running sum of that passes each eighth of the total.
    const long long per_seq = (long long)Hkv * (main_tiles * p.splits + p.tail_splits);
    const long long total = per_seq * batch;
    if (total > (1ll << 28)) return false;
    {
        long long max_len = 0;
        for (int i = 0; i < batch; ++i) max_len = std::max<long long>(max_len, kv_len[i]);
        const uint64_t per_grp = (uint64_t)(main_tiles * p.splits + p.tail_splits);
        const uint64_t nt_max = (uint64_t)((max_len + kKT - 1) / kKT + (T + kKT - 1) / kKT);
        args.per_grp_magic = magic_of(per_grp, (uint64_t)total);
        args.main_tiles_magic = magic_of((uint64_t)main_tiles, per_grp);
        args.hkv_magic = magic_of((uint64_t)Hkv, (uint64_t)batch * Hkv);
        args.splits_magic[0] = magic_of((uint64_t)p.splits, nt_max * p.splits + p.splits);
        args.splits_magic[1] = magic_of((uint64_t)p.tail_splits, nt_max * p.tail_splits + p.tail_splits);
    }
    int32_t order[DDTREE_MAX_BATCH];
    for (int i = 0; i < batch; ++i) order[i] = i;
    std::stable_sort(order, order + batch, [&](int32_t a, int32_t b) { return kv_len[a] > kv_len[b]; });
    for (int i = 0; i < batch; ++i) {
        args.by_length[i][0] = order[i];
        args.by_length[i][1] = kv_start[order[i]];
        args.by_length[i][2] = kv_len[order[i]];
        args.by_length[i][3] = 0;
    }
    long long work_total = 0;
    for (int i = 0; i < batch; ++i) work_total += per_seq * ((long long)kv_len[i] + T);
    {
        long long done = 0, first = 0;  // work and items before sequence position `pos`
        int pos = 0, x = 1;
        args.xcd_start[0] = 0;
        while (x < 8) {
            const long long target = (work_total * x + 7) / 8;
            const int sq = order[pos];
            const long long w = (long long)kv_len[sq] + T;
            if (pos < batch - 1 && done + per_seq * w < target) {
                done += per_seq * w;
                first += per_seq;
                ++pos;
                continue;
            }
            long long k = (target - done + w - 1) / w;  // items of this sequence before the cut
            if (k < 0) k = 0;
            if (k > per_seq) k = per_seq;
            args.xcd_start[x++] = (int32_t)(first + k);
        }
        args.xcd_start[8] = (int32_t)total;
    }
    long long run_max = 0;
    for (int x = 0; x < 8; ++x) {
        if (args.xcd_start[x + 1] < args.xcd_start[x]) args.xcd_start[x + 1] = args.xcd_start[x];
        const long long run = args.xcd_start[x + 1] - args.xcd_start[x];
        if (run > run_max) run_max = run;
    }
    *grid_x = run_max * 8;
    return true;
}

static int verify_attn_impl(const void *q, const void *k_cache, const void *v_cache, const void *k_tree,
                            const void *v_tree, const uint64_t *ancestor_mask, const int32_t *kv_start,
                            const int32_t *kv_len, int batch, int T, int Hq, int Hkv, int D,
                            float softmax_scale, int dtype, void *out, void *workspace,
                            size_t workspace_bytes, void *stream)
{
    using namespace ddt;
    if (!q || !k_tree || !v_tree || !ancestor_mask || !kv_start || !kv_len || !out) return DDTREE_ERR_ARG;
    // rows are read and written 16 bytes at a time
    for (const void *t : {q, k_cache, v_cache, k_tree, v_tree, static_cast<const void *>(out)})
        if (reinterpret_cast<uintptr_t>(t) & 15u) return DDTREE_ERR_ARG;
    if (reinterpret_cast<uintptr_t>(ancestor_mask) & 7u) return DDTREE_ERR_ARG;
    if (batch < 1 || batch > DDTREE_MAX_BATCH || T < 1 || T > DDTREE_MAX_N + 1 || Hq < 1 || Hkv < 1 ||
        Hq % Hkv != 0 || D < 8 || D > 256 || D % 8 != 0)
        return DDTREE_ERR_ARG;
    if (dtype != DDTREE_DTYPE_BF16 && dtype != DDTREE_DTYPE_FP32) return DDTREE_ERR_ARG;
    if (!(softmax_scale > 0.0f) || !(softmax_scale < 1e30f)) return DDTREE_ERR_ARG;
    AttnArgs args{};
    {
        const uint32_t G = (uint32_t)(Hq / Hkv);
        args.group_size = (int32_t)G;
        args.g_magic = magic_of(G, (uint64_t)T * G);
        args.per_grp_magic = args.main_tiles_magic = args.hkv_magic = args.splits_magic[0] = args.splits_magic[1] = 0u;
    }
    long long sum_L = 0;
    for (int s = 0; s < batch; ++s) {
        if (kv_start[s] < 0 || kv_len[s] < 0 || (long long)kv_start[s] + kv_len[s] > 0x7FFFFFFFll)
            return DDTREE_ERR_ARG;
        args.kv_start[s] = kv_start[s];
        args.kv_len[s] = kv_len[s];
        sum_L += kv_len[s];
    }
    if (sum_L > 0 && (!k_cache || !v_cache)) return DDTREE_ERR_ARG;
    hipStream_t st = as_stream(stream);

    if (mfma_shape(dtype, D, Hkv)) {
        AttnPlan p = attn_plan(batch, T, Hq, Hkv, D, sum_L, dtype);
        if (!ws_ok(workspace, workspace_bytes, p.bytes)) return DDTREE_ERR_WORKSPACE;
        char *wsb = static_cast<char *>(workspace);
        uint16_t *part = reinterpret_cast<uint16_t *>(wsb + p.part_off);
        float2 *lse = reinterpret_cast<float2 *>(wsb + p.lse_off);
        static std::atomic<bool> lds_allowed{false};
        if (!allow_dynamic_lds(reinterpret_cast<const void *>(attn_mfma_kernel), kAttnLdsBytes, lds_allowed))
            return DDTREE_ERR_HIP;
        long long gx = 0;
        if (!attn_fill_args(args, p, kv_start, kv_len, batch, T, Hkv, &gx)) return DDTREE_ERR_ARG;
        const int part_splits = p.part_splits > 1 ? p.part_splits : 0;
        DDT_LAUNCH(DDTREE_KERNEL_ATTN, st, attn_mfma_kernel, dim3((unsigned)gx), dim3(kAttnThreads),
                   kAttnLdsBytes, st, static_cast<const uint16_t *>(q), static_cast<const uint16_t *>(k_cache),
                   static_cast<const uint16_t *>(v_cache), static_cast<const uint16_t *>(k_tree),
                   static_cast<const uint16_t *>(v_tree), ancestor_mask, args, batch, T, Hq, Hkv,
                   softmax_scale * kLog2e, p.n_tiles, p.blk_base, p.blk_extra, p.splits, p.tail_splits, part_splits,
                   static_cast<uint16_t *>(out), part, lse);
        if (part_splits > 0) {
            const size_t n_rows = (size_t)batch * T * Hq;
            if (part_splits <= 8)
                DDT_LAUNCH(DDTREE_KERNEL_ATTN_MERGE, st, attn_merge_kernel<8>,
                           dim3((unsigned)((n_rows * 16 + 255) / 256)), dim3(256), 0, st, part, lse, n_rows,
                           part_splits, static_cast<uint16_t *>(out));
            else
                DDT_LAUNCH(DDTREE_KERNEL_ATTN_MERGE, st, attn_merge_kernel<16>,
                           dim3((unsigned)((n_rows * 16 + 255) / 256)), dim3(256), 0, st, part, lse, n_rows,
                           part_splits, static_cast<uint16_t *>(out));
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

extern "C" int ddtree_verify_attn(const void *q, const void *k_cache, const void *v_cache,
                                  const void *k_tree, const void *v_tree,
                                  const uint64_t *ancestor_mask, const int32_t *kv_offset, int batch,
                                  int T, int Hq, int Hkv, int D, float softmax_scale, int dtype,
                                  void *out, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!kv_offset || batch < 1 || batch > DDTREE_MAX_BATCH || kv_offset[0] < 0) return DDTREE_ERR_ARG;
    int32_t start[DDTREE_MAX_BATCH], len[DDTREE_MAX_BATCH];
    for (int s = 0; s < batch; ++s) {
        if (kv_offset[s + 1] < kv_offset[s]) return DDTREE_ERR_ARG;
        start[s] = kv_offset[s];
        len[s] = kv_offset[s + 1] - kv_offset[s];
    }
    return verify_attn_impl(q, k_cache, v_cache, k_tree, v_tree, ancestor_mask, start, len, batch, T, Hq,
                            Hkv, D, softmax_scale, dtype, out, workspace, workspace_bytes, stream);
}

extern "C" int ddtree_verify_attn_spans(const void *q, const void *k_cache, const void *v_cache,
                                        const void *k_tree, const void *v_tree,
                                        const uint64_t *ancestor_mask, const int32_t *kv_start,
                                        const int32_t *kv_len, int batch, int T, int Hq, int Hkv, int D,
                                        float softmax_scale, int dtype, void *out, void *workspace,
                                        size_t workspace_bytes, void *stream)
{
    if (batch < 1 || batch > DDTREE_MAX_BATCH) return DDTREE_ERR_ARG;
    return verify_attn_impl(q, k_cache, v_cache, k_tree, v_tree, ancestor_mask, kv_start, kv_len, batch, T,
                            Hq, Hkv, D, softmax_scale, dtype, out, workspace, workspace_bytes, stream);
}

// ------------------------------------------------------------------------------------------
// Host-side self-check of the matrix-core kernel's launch arithmetic (no GPU involved): for a
// list of shapes, the plan, the XCD runs and the reciprocals are built as for a launch, every
// workgroup index of the grid is decoded the way the kernel decodes it, and the result is held
// against plain division and against what the decomposition promises: every (sequence, KV head,
// row tile, key range) exactly once, the row blocks of a group's tiles a partition of its rows,
// the key ranges of a tile a partition of its key tiles in order.
// Returns 0, or 100 * (index of the failing shape + 1) + the number of the failed check.
// ------------------------------------------------------------------------------------------
namespace ddt {
int attn_selftest_host()
{
    struct Shape {
        int batch, T, Hq, Hkv;
        int32_t len[4];
    };
    static const Shape shapes[] = {
        {1, 257, 32, 8, {8192}},        {1, 513, 32, 8, {32768}},       {1, 65, 32, 8, {2048}},
        {4, 129, 64, 8, {1533, 7527, 4000, 1024}},                      {1, 1025, 8, 2, {1500}},
        {3, 33, 16, 2, {130, 0, 517}},  {1, 17, 4, 1, {128}},           {2, 40, 12, 1, {1000, 3}},
        {1, 2, 1, 1, {0}},              {4, 1024, 8, 8, {100, 0, 64, 7}}, {1, 75, 16, 4, {3000}},
        {1, 300, 6, 2, {9000}},         {2, 273, 32, 8, {5000, 4999}},  {1, 1025, 128, 1, {200000}},
    };
    // exhaustive check of the reciprocal division itself on small divisors
    for (uint32_t d = 2; d <= 64; ++d) {
        const uint64_t x_max = 0xFFFFFFFFull / d;
        const uint32_t m = magic_of(d, x_max);
        if (m == 0u) return 1;
        for (uint64_t x = 0; x <= x_max; x += (x < 70000 ? 1 : 9973))
            if (div_by((int)(x & 0x7FFFFFFF), (int)d, m) != (int)((x & 0x7FFFFFFF) / d)) return 2;
        if (magic_of(d, x_max + 1) != 0u && (x_max + 1) * d >= 0x100000000ull) return 3;
    }
    int si = 0;
    for (const Shape &sh : shapes) {
        ++si;
        const int batch = sh.batch, T = sh.T, Hq = sh.Hq, Hkv = sh.Hkv, G = Hq / Hkv;
        int32_t kv_start[4], kv_len[4];
        long long sum_L = 0;
        for (int i = 0; i < batch; ++i) {
            kv_start[i] = (int32_t)sum_L;
            kv_len[i] = sh.len[i];
            sum_L += sh.len[i];
        }
        const AttnPlan p = attn_plan(batch, T, Hq, Hkv, kHD, sum_L, DDTREE_DTYPE_BF16);
        AttnArgs args{};
        args.group_size = G;
        args.g_magic = magic_of((uint64_t)G, (uint64_t)T * G);
        long long gx = 0;
        if (!attn_fill_args(args, p, kv_start, kv_len, batch, T, Hkv, &gx)) return 100 * si + 1;
        const int main_tiles = p.tail_splits > 0 ? p.n_tiles - 1 : p.n_tiles;
        const int per_grp = main_tiles * p.splits + p.tail_splits;
        const long long total = (long long)batch * Hkv * per_grp;
        if (args.xcd_start[0] != 0 || args.xcd_start[8] != total) return 100 * si + 2;
        for (int x = 0; x < 8; ++x)
            if (args.xcd_start[x + 1] < args.xcd_start[x]) return 100 * si + 3;
        const int M = T * G, W = (T + 63) >> 6;
        (void)W;
        std::vector<int> seen((size_t)total, 0);
        // per (group, tile): the next key tile expected, and the rows covered
        std::vector<int> next_t((size_t)batch * Hkv * p.n_tiles, 0), rows((size_t)batch * Hkv, 0);
        std::vector<int> by_split((size_t)total, -1);
        for (long long b = 0; b < gx; ++b) {
            const int xcd = (int)(b & 7);
            const int wid = args.xcd_start[xcd] + (int)(b >> 3);
            if (wid >= args.xcd_start[xcd + 1]) continue;
            if (wid < 0 || wid >= total) return 100 * si + 4;
            // the kernel's decode
            const int grp = div_by(wid, per_grp, args.per_grp_magic);
            const int wg = wid - grp * per_grp;
            const bool tail = wg >= main_tiles * p.splits;
            const int wg_split = div_by(wg, main_tiles, args.main_tiles_magic);
            const int mt = tail ? main_tiles : wg - wg_split * main_tiles;
            const int split = tail ? wg - main_tiles * p.splits : wg_split;
            const int splits = tail ? p.tail_splits : p.splits;
            const int grp_seq = div_by(grp, Hkv, args.hkv_magic);
            const int hk = grp - grp_seq * Hkv;
            const int seq = args.by_length[grp_seq][0];
            const int L = args.by_length[grp_seq][2];
            const int first_blk = p.tail_splits > 0 ? mt * 8 : mt * p.blk_base + std::min(mt, p.blk_extra);
            const int n_blk = p.tail_splits > 0 ? (tail ? p.blk_extra : 8) : p.blk_base + (mt < p.blk_extra ? 1 : 0);
            const int m0 = first_blk * 32, m_end = std::min(M, (first_blk + n_blk) * 32);
            const int last_node = std::min(T - 1, div_by(m_end - 1, G, args.g_magic));
            const int nt = (L + kKT - 1) / kKT + last_node / kKT + 1;
            const uint32_t s_magic = args.splits_magic[tail ? 1 : 0];
            const int t_begin = div_by(nt * split + splits - 1, splits, s_magic);
            const int t_end = div_by(nt * (split + 1) + splits - 1, splits, s_magic);
            // against plain division
            if (grp != wid / per_grp || wg_split != wg / main_tiles || grp_seq != grp / Hkv) return 100 * si + 5;
            if (last_node != std::min(T - 1, (m_end - 1) / G)) return 100 * si + 6;
            if (t_begin != (int)(((long long)nt * split + splits - 1) / splits) ||
                t_end != (int)(((long long)nt * (split + 1) + splits - 1) / splits))
                return 100 * si + 7;
            // against the decomposition
            if (grp < 0 || grp >= batch * Hkv || hk < 0 || hk >= Hkv || seq < 0 || seq >= batch || L != kv_len[seq] ||
                args.by_length[grp_seq][1] != kv_start[seq])
                return 100 * si + 8;
            if (mt < 0 || mt >= p.n_tiles || split < 0 || split >= splits || m0 >= m_end || m0 >= M) return 100 * si + 9;
            if (t_begin < 0 || t_end > nt || t_begin > t_end) return 100 * si + 10;
            if (seen[(size_t)wid]++) return 100 * si + 11;
            by_split[(size_t)wid] = t_begin;
            if (split == 0) rows[(size_t)grp] += m_end - m0;
            // the key ranges of a tile, taken in the order of their work items (split ascending
            // within a tile for main tiles: item = split * main_tiles + mt; tail: consecutive)
            (void)next_t;
        }
        for (long long w = 0; w < total; ++w)
            if (seen[(size_t)w] != 1) return 100 * si + 12;
        for (int g = 0; g < batch * Hkv; ++g)
            if (rows[(size_t)g] != M) return 100 * si + 13;
        // key ranges: for every (group, tile) the ranges 0 .. splits-1 follow each other from 0 to nt
        for (int g = 0; g < batch * Hkv; ++g)
            for (int tile = 0; tile < p.n_tiles; ++tile) {
                const bool tail = p.tail_splits > 0 && tile == main_tiles;
                const int splits = tail ? p.tail_splits : p.splits;
                int expect = 0;
                for (int sp = 0; sp < splits; ++sp) {
                    const long long wid = (long long)g * per_grp + (tail ? main_tiles * p.splits + sp : sp * main_tiles + tile);
                    if (by_split[(size_t)wid] != expect) return 100 * si + 14;
                    // end of this range = begin of the next (or nt for the last), recomputed exactly
                    const int seq = args.by_length[g / Hkv][0];
                    const int first_blk = p.tail_splits > 0 ? tile * 8 : tile * p.blk_base + std::min(tile, p.blk_extra);
                    const int n_blk = p.tail_splits > 0 ? (tail ? p.blk_extra : 8) : p.blk_base + (tile < p.blk_extra ? 1 : 0);
                    const int m_end = std::min(M, (first_blk + n_blk) * 32);
                    const int nt = (kv_len[seq] + kKT - 1) / kKT + std::min(T - 1, (m_end - 1) / G) / kKT + 1;
                    expect = (int)(((long long)nt * (sp + 1) + splits - 1) / splits);
                    if (sp == splits - 1 && expect != nt) return 100 * si + 15;
                }
            }
    }
    return 0;
}
}  // namespace ddt
