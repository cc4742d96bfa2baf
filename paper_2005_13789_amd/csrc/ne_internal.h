// Internal declarations shared by the translation units of libne.so: handle layouts, host error
// plumbing and the small device helpers (Philox, alias draw, lane-group reductions).
#pragma once
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "ne.h"

// ---------------------------------------------------------------------------------------------
// host-side error plumbing and handles
// ---------------------------------------------------------------------------------------------
// Records the message for ne_last_error() on this thread and returns st (defined in ne.hip).
ne_status fail(ne_status st, const std::string& msg);

#define NE_HIP_CHECK(expr)                                                                       \
    do {                                                                                         \
        hipError_t e_ = (expr);                                                                  \
        if (e_ != hipSuccess)                                                                    \
            return fail(NE_ERR_HIP, std::string(#expr) + ": " + hipGetErrorString(e_));          \
    } while (0)

namespace {

// Device workspace of a tables handle (caller's memory, carved up here).
struct PrepSlot {
    unsigned long long* slots;  // [cap]  (key << 32 | reference index) per hash position; ~0 = empty
    uint8_t* shared;            // [cap]  1 <=> the row whose key sits at this position is shared
    int32_t* ids;               // [max_B][max_K+2]  src, ctx, negatives
    uint32_t* posbuf;           // [max_B][max_K+2]  final hash position of each reference
    uint8_t* refshared;         // [max_B][max_K+2]  1 <=> another reference of the batch names this reference's row too
};
struct Workspace {
    PrepSlot prep[2];
    float* delta;        // [cap][dim]  per-position fp32 accumulators, zero between batches
    uint32_t* count;     // [cap]       arrivals at a shared row's position, zero between batches
    uint32_t* members;   // [cap][8]    reference indices of a shared row's first arrivals
    float* dbuf;         // [max_B * (max_K + 2)][dim]  per-reference deltas of those arrivals
    uint32_t cap;        // power of two >= 2 * max_B * (max_K + 2)
    size_t total_bytes;
};

}  // namespace

struct ne_tables {
    int64_t num_nodes;
    int32_t dim;
    float* vertex;
    float* context;
    uint64_t seed;
    int64_t max_batch;
    int32_t max_negatives;
    Workspace ws;
    uint64_t batches_done;
    bool workspace_dirty;    // a launch failed in the middle of a run of batches: hash state, flags and slots may be half-used
    int32_t tune_list_cap;   // ne_set_tuning: -1 = automatic
    int32_t tune_sweep;      // ne_set_tuning: 0 = automatic
    // optional timing of the train kernel with HIP events (ne_profile_enable / ne_profile_read)
    int32_t profile_every;
    std::vector<hipEvent_t> ev_zero, ev_start, ev_stop;   // zero -> start brackets nothing: the events' own cost
    size_t ev_used;
};

struct ne_alias {
    const uint2* table;  // device {threshold, alias}[n]
    int64_t n;
    int32_t base;
};

// Timing of one kernel with HIP events.  profile_begin records two events back to back (the gap
// between them is what recording costs on this stream) and profile_end a third after the kernel.
inline bool profile_begin(ne_tables* t, hipStream_t st)
{
    const bool timed = t->profile_every > 0 && t->batches_done % static_cast<uint64_t>(t->profile_every) == 0 &&
                       t->ev_used < t->ev_start.size();
    if (!timed) return false;
    if (hipEventRecord(t->ev_zero[t->ev_used], st) != hipSuccess) return false;
    return hipEventRecord(t->ev_start[t->ev_used], st) == hipSuccess;
}

inline void profile_end(ne_tables* t, hipStream_t st)
{
    if (hipEventRecord(t->ev_stop[t->ev_used], st) == hipSuccess) t->ev_used += 1;
}

// Home position of a row key in a table of mask + 1 positions (a power of two, at most 2^31): the top
// log2(positions) bits of a Fibonacci multiplicative hash, so that every position is some key's home
// however large the table (a fixed shift would leave tables wider than its bits mostly unreachable and
// pile the keys into one cluster).
__host__ __device__ __forceinline__ uint32_t hash_position(uint32_t key, uint32_t mask)
{
#if defined(__HIP_DEVICE_COMPILE__)
    const int shift = __clz(static_cast<int>(mask));
#else
    const int shift = __builtin_clz(mask);
#endif
    return (key * 0x9E3779B1u) >> shift;
}

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// ---------------------------------------------------------------------------------------------
// device helpers
// ---------------------------------------------------------------------------------------------
namespace {

enum : uint32_t { kStreamNegative = 0, kStreamInit = 1, kStreamSharedNegative = 2 };

// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11).
__device__ __forceinline__ uint4 philox4x32_10(uint4 c, uint32_t k0, uint32_t k1)
{
    constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    constexpr uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(M0, c.x), lo0 = M0 * c.x;
        const uint32_t hi1 = __umulhi(M1, c.z), lo1 = M1 * c.z;
        c = make_uint4(hi1 ^ c.y ^ k0, lo1, hi0 ^ c.w ^ k1, lo0);
        k0 += W0;
        k1 += W1;
    }
    return c;
}

// One alias draw: slot = floor(((r0<<32)|r1) * n / 2^64); keep slot iff r2 < threshold[slot].
__device__ __forceinline__ int32_t alias_draw(uint4 r, const uint2* __restrict__ table, uint64_t n)
{
    const uint64_t u = (static_cast<uint64_t>(r.x) << 32) | r.y;
    const uint64_t slot = __umul64hi(u, n);
    const uint2 e = table[slot];
    return static_cast<int32_t>(r.z < e.x ? static_cast<uint32_t>(slot) : e.y);
}

__device__ __forceinline__ int32_t draw_negative(uint64_t sample, uint32_t k, uint32_t k0, uint32_t k1,
                                                 const uint2* __restrict__ table, uint64_t n, int32_t base)
{
    const uint4 r = philox4x32_10(make_uint4(static_cast<uint32_t>(sample), static_cast<uint32_t>(sample >> 32), k,
                                             kStreamNegative), k0, k1);
    return base + alias_draw(r, table, n);
}

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}

// Sum over the G lanes of a lane group (G = 8, 16, 32 or 64, groups aligned to G); every lane of
// the group ends with the total.  Lanes 1, 2 apart: DPP quad permutes; 4, 8 apart: DPP half-row and
// row mirrors (valid because the partial sums are already equal inside each quad / half row);
// 16 apart: ds_swizzle; 32 apart: ds_bpermute.
template <int G>
__device__ __forceinline__ float group_sum(float v)
{
    v += dpp_move<0xB1>(v);   // quad_perm [1,0,3,2]
    v += dpp_move<0x4E>(v);   // quad_perm [2,3,0,1]
    v += dpp_move<0x141>(v);  // row_half_mirror
    if (G >= 16) v += dpp_move<0x140>(v);  // row_mirror
    if (G >= 32) v += __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(v), 0x401F));  // lane ^ 16
    if (G >= 64) v += __shfl_xor(v, 32, 64);
    return v;
}

__device__ __forceinline__ float sigmoidf(float z) { return 1.0f / (1.0f + expf(-z)); }
__device__ __forceinline__ float softplusf(float z) { return fmaxf(z, 0.0f) + log1pf(expf(-fabsf(z))); }

__device__ __forceinline__ float dot4(float4 a, float4 b)
{
    return fmaf(a.x, b.x, fmaf(a.y, b.y, fmaf(a.z, b.z, a.w * b.w)));
}

__device__ __forceinline__ float4 axpy4(float g, float4 x, float4 y)
{
    return make_float4(fmaf(g, x.x, y.x), fmaf(g, x.y, y.y), fmaf(g, x.z, y.z), fmaf(g, x.w, y.w));
}

}  // namespace
