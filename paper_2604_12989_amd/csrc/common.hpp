// Shared device/host helpers for the gfx950 kernels of the DDTree draft-tree step.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

#include "ddtree.h"

namespace ddt {

constexpr int kWave = 64;

inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

inline int launch_status()
{
    return hipGetLastError() == hipSuccess ? DDTREE_OK : DDTREE_ERR_HIP;
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Raises a kernel's dynamic-LDS limit, once per process.  The call is idempotent, so two host
// threads that race here simply both make it.  False if the runtime refuses.
inline bool allow_dynamic_lds(const void *kernel, size_t bytes, std::atomic<bool> &done)
{
    if (done.load(std::memory_order_acquire)) return true;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess)
        return false;
    done.store(true, std::memory_order_release);
    return true;
}
inline bool ws_ok(const void *ws, size_t have, size_t need)
{
    return need == 0 || (ws != nullptr && (reinterpret_cast<uintptr_t>(ws) & 255u) == 0 && have >= need);
}

// ---- layout of the top-K scratch, shared by the host sizing code and the kernels ----
struct TopkPlan {
    int chunks;     // chunks per logits row
    int chunk_len;  // elements per chunk (multiple of 4), last chunk may be shorter
    int kc;         // candidates kept per chunk = min(K, chunk_len)
    size_t cand_off, stat_off, bytes;
    bool ok;
    bool row_kernel;  // many rows: one workgroup scans a whole row, no chunks and no scratch
};
constexpr int kTopkRowKernelMinRows = 128;
constexpr int kTopkChunkMax = 12288;      // keys held in LDS by one chunk workgroup
constexpr int kTopkMergeMaxCand = 14336;  // u64 candidates held in LDS by the merge workgroup
TopkPlan topk_plan(int batch, int B, int V, int K);

// ---- layout of the attention scratch ----
struct AttnPlan {
    // The query rows of one (sequence, kv head) pair, in blocks of 32, are dealt as evenly as
    // possible to n_tiles row tiles of at most 8 blocks: tile i holds blk_base + (i < blk_extra)
    // blocks.  The key range of every tile is cut into `splits` parts; partial results exist
    // only when splits > 1.
    int n_tiles, blk_base, blk_extra, splits;
    // Uneven form (tail_splits > 0): the first n_tiles - 1 tiles hold 8 blocks and `splits` key
    // ranges each; the last tile holds the few blocks left over (at most one wave per SIMD, so
    // it runs about twice as fast per key tile) and `tail_splits` key ranges.  Partials are laid
    // out for part_splits = max(splits, tail_splits) ranges.
    int tail_splits, part_splits;
    size_t part_off, lse_off, bytes;
};
AttnPlan attn_plan(int batch, int T, int Hq, int Hkv, int D, long long sum_L, int dtype);

// ---- layout of the accept scratch ----
struct AcceptPlan {
    int splits;  // segments per logits row
    int seg_len; // elements per segment (multiple of 4)
    size_t part_off, bytes;
};
AcceptPlan accept_plan(int batch, int T, int V, bool sampled = false);  // the greedy plan needs the larger scratch

// ---- optional event timing around kernel launches (see ddtree_profile_enable) ----
struct Profiler {
    unsigned mask = 0;
    int capacity = 0;
    int every = 1;                          // time one launch in `every`
    int seen[DDTREE_KERNEL_COUNT] = {};     // launches since the hook was switched on
    int count[DDTREE_KERNEL_COUNT] = {};
    hipEvent_t *start[DDTREE_KERNEL_COUNT] = {};
    hipEvent_t *stop[DDTREE_KERNEL_COUNT] = {};
};
Profiler &profiler();
// The slot that times this launch of kernel `id`, or -1 if the launch is not timed.
inline int profile_slot(int id)
{
    Profiler &p = profiler();
    if (!(p.mask & (1u << id)) || p.count[id] >= p.capacity) return -1;
    if (p.seen[id]++ % p.every != 0) return -1;
    return p.count[id]++;
}
// A timed launch hands its two events to the launch itself: they take the begin and end time
// stamps of the dispatch, with no marker packets of their own on the stream (a pair of recorded
// events reads about 5 us with nothing between them, and delays the kernels around it).
#define DDT_LAUNCH(id, st, kernel, grid, block, lds, stream, ...)                                    \
    do {                                                                                             \
        const int _slot = ::ddt::profile_slot(id);                                                   \
        if (_slot < 0)                                                                               \
            hipLaunchKernelGGL(kernel, grid, block, lds, stream, __VA_ARGS__);                       \
        else                                                                                         \
            hipExtLaunchKernelGGL(kernel, grid, block, lds, stream, ::ddt::profiler().start[id][_slot], \
                                  ::ddt::profiler().stop[id][_slot], 0, __VA_ARGS__);                 \
    } while (0)

#if defined(__HIPCC__)
// Order-preserving map from finite floats to unsigned integers (-0 is folded onto +0).
__device__ __forceinline__ uint32_t float_key(float x)
{
    uint32_t b = __float_as_uint(x);
    if (b == 0x80000000u) b = 0u;
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float key_float(uint32_t k)
{
    uint32_t b = (k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k;
    return __uint_as_float(b);
}

// Wave-wide max of a float over all 64 lanes via DPP, returned uniformly.
// All 64 lanes must be active.
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ float dpp_f(float old, float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(old), __float_as_int(v), CTRL,
                                                      ROW_MASK, 0xF, false));
}
__device__ __forceinline__ float wave_max_f32(float v)
{
    v = fmaxf(v, dpp_f<0xB1>(v, v));   // quad_perm [1,0,3,2]
    v = fmaxf(v, dpp_f<0x4E>(v, v));   // quad_perm [2,3,0,1]
    v = fmaxf(v, dpp_f<0x141>(v, v));  // row_half_mirror
    v = fmaxf(v, dpp_f<0x140>(v, v));  // row_mirror: every lane of a 16-lane row holds the row max
    v = fmaxf(v, dpp_f<0x142, 0xA>(v, v));  // row_bcast15 into rows 1 and 3
    v = fmaxf(v, dpp_f<0x143, 0xC>(v, v));  // row_bcast31 into rows 2 and 3
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// Wave-wide minimum of an unsigned value over all 64 lanes (all lanes must be active).
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ uint32_t dpp_u(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, ROW_MASK, 0xF, false);
}
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v)
{
    v = min(v, dpp_u<0xB1>(v));
    v = min(v, dpp_u<0x4E>(v));
    v = min(v, dpp_u<0x141>(v));
    v = min(v, dpp_u<0x140>(v));
    v = min(v, dpp_u<0x142, 0xA>(v));
    v = min(v, dpp_u<0x143, 0xC>(v));
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

// DPP move that leaves 0 in lanes with no source lane (or in rows outside ROW_MASK).
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ int dpp_or_zero(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, CTRL, ROW_MASK, 0xF, false);
}
// Inclusive prefix sum over the wave's 64 lanes (all lanes must be active).
__device__ __forceinline__ int wave_scan_inclusive_i32(int v)
{
    v += dpp_or_zero<0x111>(v);  // row_shr:1
    v += dpp_or_zero<0x112>(v);  // row_shr:2
    v += dpp_or_zero<0x114>(v);  // row_shr:4
    v += dpp_or_zero<0x118>(v);  // row_shr:8  -> inclusive inside each row of 16
    v += dpp_or_zero<0x142, 0xA>(v);  // rows 1 and 3 add the total of the row before
    v += dpp_or_zero<0x143, 0xC>(v);  // rows 2 and 3 add the total of rows 0-1
    return v;
}
// Sum of a double over the wave in a fixed order; the result is valid in lane 63 only.
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ double dpp_d_or_zero(double v)
{
    const int lo = dpp_or_zero<CTRL, ROW_MASK>(__double2loint(v));
    const int hi = dpp_or_zero<CTRL, ROW_MASK>(__double2hiint(v));
    return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double wave_sum_f64_lane63(double v)
{
    v += dpp_d_or_zero<0xB1>(v);
    v += dpp_d_or_zero<0x4E>(v);
    v += dpp_d_or_zero<0x141>(v);
    v += dpp_d_or_zero<0x140>(v);
    v += dpp_d_or_zero<0x142, 0xA>(v);
    v += dpp_d_or_zero<0x143, 0xC>(v);
    return v;
}

__device__ __forceinline__ int lane_id() { return __lane_id(); }
#endif

}  // namespace ddt
