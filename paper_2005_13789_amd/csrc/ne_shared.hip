// Shared-negative SGNS step for MI355X (gfx950): ne_train_batch_shared.
//
// All B pairs of a batch are scored against the same N negative rows, which turns scoring and both
// gradient products into dense contractions (the level-3 formulation the paper cites as related
// work, Sec. VI-B):
//     S  = Xq . Cq^T            [B x d] . [d x N]      scores
//     G  = -neg_scale sigma(S)                          coefficients (rounded to bf16)
//     dX = G . Cq               [B x N] . [N x d]      gradient of the source rows
//     dC = G^T . Xq             [N x B] . [B x d]      gradient of the negative rows
// with Xq, Cq the gathered rows rounded to bf16 and fp32 accumulation on the matrix cores
// (v_mfma_f32_32x32x16_bf16).  The positive pair of every sample is handled in full fp32.
//
// Four kernels per batch; the tables are only read by the first two and only written by the last:
//   prep    draws the N negatives, gathers their rows, rounds them and stores them twice in the order
//           in which the matrix-core operands of the two products want them (one coalesced 1 KB read per
//           operand fragment later); claims every row reference of the batch (plain-store hashing).
//   scores  one workgroup per 32 pairs, all N negatives: gathers its pairs' rows, does the positive
//           pairs in fp32, S block by block on MFMA with the negatives' fragments streamed from
//           memory (they stay in L2), sigmoid in registers, G to LDS (and transposed to memory for the
//           dC product), dX accumulated on MFMA over all negatives: a workgroup ends with the complete
//           deltas of its pairs' source rows, no partial sums.  The resolve pass rides along.
//   dctx    dC = G^T . Xq on MFMA, split over the batch dimension into partial sums.
//   update  adds every staged delta to the tables.  Nothing reads the tables any more at that point,
//           so duplicates simply add up: rows named once in the batch are rewritten with plain stores,
//           the others take fp32 atomics.
#include <hip/hip_bf16.h>

#include <mutex>

#include "ne_internal.h"

// Workspace of ne_train_batch_shared_static: one array per GPU, part of the loaded code object, so the
// entry point has nothing to allocate.  The name below is only a host-side stand-in; the device
// address comes from hipGetSymbolAddress (static_scratch_of_current_device) and is what the kernels get.
constexpr size_t kStaticScratchBytes = static_cast<size_t>(NE_SHARED_STATIC_SCRATCH_BYTES);
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kPairTile = 32;      // pairs per workgroup in the scores kernel
constexpr int kScoreThreads = 512; // 8 wavefronts: one 32-negative block of S each, one 32-column block of dX each
constexpr int kNegChunk = 256;     // negatives per pass of the scores kernel (8 wavefronts x 32)
constexpr int kSplit = 16;         // partial sums of the dC product
constexpr int kBatchPad = 1024;    // the padded batch is a multiple of this (kSplit shares of whole 64-pair steps)

__device__ __forceinline__ uint16_t to_bf16(float x)
{
    uint32_t u = __float_as_uint(x);
    u += 0x7FFFu + ((u >> 16) & 1u);   // round to nearest even
    return static_cast<uint16_t>(u >> 16);
}

// sigmoid from the hardware exp2 and reciprocal (about 1 ulp each): the result is rounded to bf16 anyway
__device__ __forceinline__ float fast_sigmoidf(float z) { return __frcp_rn(1.0f + __expf(-z)); }

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

// Workgroup barrier for data exchanged through LDS only: waits for this wavefront's LDS operations, not for its
// global loads and stores.  (__syncthreads also drains those, which would undo every operand fetch issued ahead of
// its use and expose the latency of every store.)
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// MFMA 32x32x16 operand layout (checked on hardware): lane l supplies row (A) / column (B) l%32 and the 8
// consecutive contraction indices (l/32)*8..+7 of the step; accumulator element i is row
// (i/4)*8 + (l/32)*4 + i%4, column l%32.  A "fragment" below is what the 64 lanes of a wavefront supply
// for one step: 64 x 8 bf16 = 1 KB, stored lane after lane.
struct SharedWs {
    uint16_t* XqT;   // [d][Bp]   bf16 source rows, transposed (zero beyond B): operand of the dC product
    uint16_t* CqP;   // [N/32][d/16][64][8]  bf16 negative rows as B fragments of S: block of 32 negatives, step over d
    uint16_t* CqTP;  // [d/32][N/16][64][8]  the same rows as B fragments of dX: block of 32 columns, step over negatives
    uint16_t* GT;    // [N][Bp]   bf16 coefficients, transposed
    float* dxs;      // [Bp][d]   complete delta of pair b's source row: lr * (g0 * c_ctx + (G . Cq)_b)
    float* dcs;      // [Bp][d]   lr * g0 * x: delta of pair b's context row
    float* dCp;      // [kSplit][N][d] partial sums of G^T . Xq
    int32_t* negids; // [N]
    unsigned long long* slots;   // [hash_mask + 1]  (key << 32 | reference) of the reference that claimed a position last
    uint8_t* multi;              // [hash_mask + 1]  1 = the row that owns this position is named more than once
    uint32_t hash_mask;
    int64_t Bp;
    size_t total;
};

// References of a batch: 2b the source row of pair b, 2b + 1 its context row, 2B + j negative j.
// key = row | (context table ? 1 << 31 : 0).
__device__ __forceinline__ uint32_t ref_hash(uint32_t key, uint32_t mask) { return hash_position(key, mask); }
__device__ __forceinline__ unsigned long long ref_entry(uint32_t key, uint32_t ref) { return (static_cast<unsigned long long>(key) << 32) | ref; }
constexpr uint32_t kContextKey = 0x80000000u;

bool shared_layout(int32_t dim, int64_t B, int32_t N, char* base, SharedWs* w)
{
    if (!(dim == 64 || dim == 128 || dim == 256) || B < 1 || B > (1 << 20) || N < 128 || N > 65536 || N % 128 != 0)
        return false;
    const size_t Bp = static_cast<size_t>((B + kBatchPad - 1) / kBatchPad) * kBatchPad;
    auto up = [](size_t v) { return (v + 255) & ~static_cast<size_t>(255); };
    size_t off = 0;
    auto take = [&](size_t bytes) { char* p = base + off; off = up(off + bytes); return p; };
    const size_t d = static_cast<size_t>(dim), n = static_cast<size_t>(N);
    w->Bp = static_cast<int64_t>(Bp);
    w->XqT = reinterpret_cast<uint16_t*>(take(Bp * d * 2));
    w->CqP = reinterpret_cast<uint16_t*>(take(n * d * 2));
    w->CqTP = reinterpret_cast<uint16_t*>(take(n * d * 2));
    w->GT = reinterpret_cast<uint16_t*>(take(n * Bp * 2));
    w->dxs = reinterpret_cast<float*>(take(Bp * d * 4));
    w->dcs = reinterpret_cast<float*>(take(Bp * d * 4));
    w->dCp = reinterpret_cast<float*>(take(static_cast<size_t>(kSplit) * n * d * 4));
    w->negids = reinterpret_cast<int32_t*>(take(n * 4));
    size_t cap = 4096;
    while (cap < 4 * (2 * Bp + n)) cap <<= 1;
    w->hash_mask = static_cast<uint32_t>(cap - 1);
    w->slots = reinterpret_cast<unsigned long long*>(take(cap * 8));
    w->multi = reinterpret_cast<uint8_t*>(take(cap));
    w->total = off;
    return true;
}

// ---------------------------------------------------------------------------------------------
// prep kernel.  Threads [0, N * G), in lane groups of G = D/8: negative j of the batch: draw its id, claim
// its row, gather the row, round it, store its 8-element pieces at their places in the two fragment
// orders.  Threads [0, 2B): claim reference t of the pairs.  All threads: clear 16 of the
// "named more than once" flags.
// ---------------------------------------------------------------------------------------------
struct PrepNegArgs {
    const float4* C;
    const int2* pairs;
    int64_t B;
    int32_t N;
    uint64_t batch_index;
    uint32_t k0, k1;
    const uint2* alias;
    uint64_t alias_n;
    int32_t alias_base;
    SharedWs w;
    int32_t* neg_out;
};

__device__ __forceinline__ uint32_t pack2(float a, float b) { return to_bf16(a) | (static_cast<uint32_t>(to_bf16(b)) << 16); }

template <int D>
__global__ __launch_bounds__(256) void prep_kernel(PrepNegArgs a)
{
    constexpr int G = D / 8;
    const int64_t t = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    // the flags start from zero in every batch
    {
        const size_t i = static_cast<size_t>(t) * 16;
        if (i <= a.w.hash_mask) *reinterpret_cast<uint4*>(a.w.multi + i) = make_uint4(0u, 0u, 0u, 0u);
    }
    // claim: whichever reference stores last owns the position of its row's key
    if (t < 2 * a.B) {
        const int2 pr = a.pairs[t >> 1];
        const uint32_t key = (t & 1) ? (static_cast<uint32_t>(pr.y) | kContextKey) : static_cast<uint32_t>(pr.x);
        a.w.slots[ref_hash(key, a.w.hash_mask)] = ref_entry(key, static_cast<uint32_t>(t));
    }
    const int64_t j64 = t / G;
    if (j64 >= a.N) return;
    const int j = static_cast<int>(j64), lg = static_cast<int>(t - j64 * G);
    const uint4 r = philox4x32_10(make_uint4(static_cast<uint32_t>(a.batch_index), static_cast<uint32_t>(a.batch_index >> 32),
                                             static_cast<uint32_t>(j), kStreamSharedNegative), a.k0, a.k1);
    const int32_t id = a.alias_base + alias_draw(r, a.alias, a.alias_n);
    if (lg == 0) {
        a.w.negids[j] = id;
        if (a.neg_out) a.neg_out[j] = id;
        const uint32_t key = static_cast<uint32_t>(id) | kContextKey;
        a.w.slots[ref_hash(key, a.w.hash_mask)] = ref_entry(key, static_cast<uint32_t>(2 * a.B + j));
    }
    // elements 8 lg .. 8 lg + 7 of the row
    const float4* crow = a.C + static_cast<int64_t>(id) * (D / 4);
    const float4 c0 = crow[2 * lg], c1 = crow[2 * lg + 1];
    const uint4 piece = make_uint4(pack2(c0.x, c0.y), pack2(c0.z, c0.w), pack2(c1.x, c1.y), pack2(c1.z, c1.w));
    // S fragments: block j / 32, step over d = lg / 2, lane = j % 32 + 32 * (lg % 2): the piece is the lane's 16 bytes
    {
        const size_t lane = static_cast<size_t>(j & 31) + 32u * (lg & 1);
        const size_t frag = static_cast<size_t>(j >> 5) * (D / 16) + (lg >> 1);
        *reinterpret_cast<uint4*>(a.w.CqP + (frag * 64 + lane) * 8) = piece;
    }
    // dX fragments: column c = 8 lg + e: block c / 32, step over negatives = j / 16, lane = c % 32 + 32 * ((j % 16) / 8),
    // element j % 8 of the lane's 8
    {
        const uint16_t h[8] = {static_cast<uint16_t>(piece.x), static_cast<uint16_t>(piece.x >> 16), static_cast<uint16_t>(piece.y),
                               static_cast<uint16_t>(piece.y >> 16), static_cast<uint16_t>(piece.z), static_cast<uint16_t>(piece.z >> 16),
                               static_cast<uint16_t>(piece.w), static_cast<uint16_t>(piece.w >> 16)};
        const size_t steps = static_cast<size_t>(a.N) / 16;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int c = 8 * lg + e;
            const size_t lane = static_cast<size_t>(c & 31) + 32u * ((j >> 3) & 1);
            const size_t frag = static_cast<size_t>(c >> 5) * steps + (j >> 4);
            a.w.CqTP[(frag * 64 + lane) * 8 + (j & 7)] = h[e];
        }
    }
}

// ---------------------------------------------------------------------------------------------
// scores kernel: one workgroup (8 wavefronts) per 32 pairs, all N negatives.
//   prologue   16 lanes per pair: gather x = vertex[src] and c = context[ctx] in fp32, positive score,
//              g0 = lr (1 - sigma(s0)); lr g0 x goes to dcs, lr g0 c stays in registers; x rounded to bf16
//              into LDS (and, transposed, to memory for the dC product); every wavefront then keeps the
//              A fragments of the 32 rows (all of d) in registers.
//   per pass of 256 negatives
//     S      wavefront w: 32 pairs x negatives block w of the pass; B fragments straight from memory.
//            G = -neg_scale sigma(S) as bf16 into LDS [32][256].
//     G^T    256 negatives x 32 pairs to memory, 64 contiguous bytes per negative.
//     dX     wavefront w: 32 pairs x columns block w (32 of d): A fragments from G in LDS, B fragments
//            straight from memory.
//   epilogue   dX through LDS to the pairs' lanes: dxs = lr dX + lr g0 c.
// ---------------------------------------------------------------------------------------------
struct ScoresArgs {
    const float4* X;
    const float4* C;
    SharedWs w;
    int64_t B;
    int32_t N;
    float lr;
    float neg_scale;
    double* loss;
    const int2* pairs;
};

template <int D, bool LOSS>
__global__ __launch_bounds__(kScoreThreads) void scores_kernel(ScoresArgs a)
{
    constexpr int XP = D + 8;            // pitch of the bf16 source rows in LDS (16-byte fragment reads spread over the banks)
    constexpr int GP = kNegChunk + 8;    // pitch of G
    constexpr int DP = D + 4;            // pitch of the fp32 dX rows
    constexpr int KS = D / 16;           // contraction steps of S
    constexpr int CB = D / 32;           // 32-column blocks of dX: wavefronts 0 .. CB-1 take one each
    constexpr int NCH = D / 64;          // float4 chunks of a row per lane of a pair's 16 lanes
    constexpr int kXsBytes = kPairTile * XP * 2, kGsBytes = kPairTile * GP * 2, kDxBytes = kPairTile * DP * 4;
    __shared__ __align__(16) unsigned char lds_raw[(kXsBytes + kGsBytes > kDxBytes) ? kXsBytes + kGsBytes : kDxBytes];
    uint16_t* Xs = reinterpret_cast<uint16_t*>(lds_raw);                    // [32][XP]
    uint16_t* Gs = reinterpret_cast<uint16_t*>(lds_raw + kXsBytes);         // [32][GP]
    float* dXs = reinterpret_cast<float*>(lds_raw);                         // [32][DP], after the last pass
    const int tid = threadIdx.x;
    const int l = tid & 63, w = tid >> 6;
    const int64_t b0 = static_cast<int64_t>(blockIdx.x) * kPairTile;
    const int64_t Bp = a.w.Bp;

    // resolve (ids only, a by-product of this launch): a reference that finds its row's key at the
    // key's position under another reference's name flags the row as named more than once
    {
        const int64_t refs = 2 * a.B + a.N;
        const int64_t stride = static_cast<int64_t>(gridDim.x) * kScoreThreads;
        for (int64_t r = static_cast<int64_t>(blockIdx.x) * kScoreThreads + tid; r < refs; r += stride) {
            uint32_t key;
            if (r < 2 * a.B) {
                const int2 pr = a.pairs[r >> 1];
                key = (r & 1) ? (static_cast<uint32_t>(pr.y) | kContextKey) : static_cast<uint32_t>(pr.x);
            } else {
                key = static_cast<uint32_t>(a.w.negids[r - 2 * a.B]) | kContextKey;
            }
            const uint32_t pos = ref_hash(key, a.w.hash_mask);
            const unsigned long long owner = a.w.slots[pos];
            if (static_cast<uint32_t>(owner >> 32) == key && static_cast<uint32_t>(owner) != static_cast<uint32_t>(r)) a.w.multi[pos] = 1;
        }
    }

    // ---- prologue: the positive pairs, in fp32
    const int p = tid >> 4, lp = tid & 15;           // pair of the tile, lane of the pair
    const int64_t b = b0 + p;
    const bool live = b < a.B;
    float4 dxp[NCH];                                 // lr g0 c
    float loss = 0.0f;
    {
        float4 x[NCH], c[NCH];
        float s0 = 0.0f;
        if (live) {
            const int2 pr = a.pairs[b];
            const float4* xrow = a.X + static_cast<int64_t>(pr.x) * (D / 4);
            const float4* crow = a.C + static_cast<int64_t>(pr.y) * (D / 4);
#pragma unroll
            for (int i = 0; i < NCH; ++i) { x[i] = xrow[lp + 16 * i]; c[i] = crow[lp + 16 * i]; }
#pragma unroll
            for (int i = 0; i < NCH; ++i) s0 += dot4(x[i], c[i]);
        } else {
#pragma unroll
            for (int i = 0; i < NCH; ++i) { x[i] = make_float4(0.f, 0.f, 0.f, 0.f); c[i] = x[i]; }
        }
        s0 = group_sum<16>(s0);
        const float g0 = live ? a.lr * (1.0f - sigmoidf(s0)) : 0.0f;
        if (LOSS && live && lp == 0) loss = softplusf(-s0);
        float4* dcs = reinterpret_cast<float4*>(a.w.dcs + b * D);
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int ci = lp + 16 * i;
            dxp[i] = make_float4(g0 * c[i].x, g0 * c[i].y, g0 * c[i].z, g0 * c[i].w);
            if (live) dcs[ci] = make_float4(g0 * x[i].x, g0 * x[i].y, g0 * x[i].z, g0 * x[i].w);
            *reinterpret_cast<uint2*>(Xs + p * XP + 4 * ci) = make_uint2(pack2(x[i].x, x[i].y), pack2(x[i].z, x[i].w));   // padding rows: zero
        }
    }
    __syncthreads();
    // by-product: the transposed copy the dC product reads, 64 contiguous bytes per column
    if (tid < D) {
        uint4* out = reinterpret_cast<uint4*>(a.w.XqT + static_cast<int64_t>(tid) * Bp + b0);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            uint32_t v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                v[i] = Xs[(8 * q + 2 * i) * XP + tid] | (static_cast<uint32_t>(Xs[(8 * q + 2 * i + 1) * XP + tid]) << 16);
            out[q] = make_uint4(v[0], v[1], v[2], v[3]);
        }
    }
    f32x16 acc_dx;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc_dx[i] = 0.0f;
    const uint4* SP = reinterpret_cast<const uint4*>(a.w.CqP);     // one uint4 per lane and fragment
    const uint4* TP = reinterpret_cast<const uint4*>(a.w.CqTP);
    const int steps_all = a.N / 16;                                // contraction steps of dX over all negatives
    // A fragments of S: row l % 32, contraction indices 16 s + 8 (l / 32) ..; A fragments of dX: the same of G
    const uint16_t* xa = Xs + (l & 31) * XP + 8 * (l >> 5);
    const uint16_t* ga = Gs + (l & 31) * GP + 8 * (l >> 5);

    // The operand fragments come straight from memory (L2: every workgroup streams the same 2 N d bytes), 1 KB per
    // wavefront and step, and each wavefront has only one other on its SIMD to hide their latency: so they are
    // requested as early as their registers are free: those of a pass's dX product and those of the next pass's S
    // product as soon as the S product has consumed its own.
    uint4 bS[KS];
    if (w * 32 < a.N) {
        const uint4* src = SP + static_cast<size_t>(w) * KS * 64 + l;
#pragma unroll
        for (int s = 0; s < KS; ++s) bS[s] = src[s * 64];
    }
    for (int n0 = 0; n0 < a.N; n0 += kNegChunk) {
        const int nblock = (n0 >> 5) + w;                 // this wavefront's block of 32 negatives (whole blocks: N % 128 == 0)
        const bool s_active = nblock * 32 < a.N;
        const bool x_active = w < CB;                     // this wavefront has a block of 32 columns of dX
        const int steps = min(kNegChunk / 16, steps_all - (n0 >> 4));   // 16, or 8 in a last pass of 128 negatives
        const uint4* tsrc = TP + (static_cast<size_t>(w) * steps_all + (n0 >> 4)) * 64 + l;
        uint4 bT0[8], bT1[8];
        f32x16 sacc;
        if (s_active) {
#pragma unroll
            for (int i = 0; i < 16; ++i) sacc[i] = 0.0f;
#pragma unroll
            for (int s = 0; s < KS; ++s)
                sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(*reinterpret_cast<const uint4*>(xa + 16 * s)), as_bf16x8(bS[s]), sacc, 0, 0, 0);
        }
        if (x_active) {                                   // (after the S product: waits on loads are in issue order)
#pragma unroll
            for (int s = 0; s < 8; ++s) bT0[s] = tsrc[s * 64];
            if (steps > 8) {
#pragma unroll
                for (int s = 0; s < 8; ++s) bT1[s] = tsrc[(8 + s) * 64];
            }
        }
        if (n0 + kNegChunk + w * 32 < a.N) {              // the S operands of the next pass
            const uint4* src = SP + static_cast<size_t>(nblock + kNegChunk / 32) * KS * 64 + l;
#pragma unroll
            for (int s = 0; s < KS; ++s) bS[s] = src[s * 64];
        }
        if (s_active) {
            // G = -neg_scale * sigmoid(S), zero for padding rows; into LDS as bf16
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int row = (i >> 2) * 8 + (l >> 5) * 4 + (i & 3);
                const bool valid = b0 + row < a.B;
                const float g = valid ? -a.neg_scale * fast_sigmoidf(sacc[i]) : 0.0f;
                if (LOSS && valid) loss += a.neg_scale * softplusf(sacc[i]);
                Gs[row * GP + w * 32 + (l & 31)] = to_bf16(g);
            }
        }
        lds_barrier();
        // G^T to memory: one negative of the pass per two threads, 16 pairs (32 bytes) each
        {
            const int neg = tid >> 1, half = tid & 1;
            if (n0 + neg < a.N) {
                uint32_t v[8];
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    v[i] = Gs[(half * 16 + 2 * i) * GP + neg] | (static_cast<uint32_t>(Gs[(half * 16 + 2 * i + 1) * GP + neg]) << 16);
                uint4* out = reinterpret_cast<uint4*>(a.w.GT + static_cast<int64_t>(n0 + neg) * Bp + b0 + half * 16);
                out[0] = make_uint4(v[0], v[1], v[2], v[3]);
                out[1] = make_uint4(v[4], v[5], v[6], v[7]);
            }
        }
        // dX += G . Cq for this wavefront's block of 32 columns over the negatives of the pass
        if (x_active) {
#pragma unroll
            for (int s = 0; s < 8; ++s)
                acc_dx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(*reinterpret_cast<const uint4*>(ga + 16 * s)), as_bf16x8(bT0[s]), acc_dx, 0, 0, 0);
            if (steps > 8) {
#pragma unroll
                for (int s = 0; s < 8; ++s)
                    acc_dx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(*reinterpret_cast<const uint4*>(ga + 16 * (8 + s))), as_bf16x8(bT1[s]), acc_dx, 0, 0, 0);
            }
        }
        lds_barrier();   // G is rewritten by the next pass (and the rows' LDS by the epilogue)
    }

    // ---- epilogue: dX to the pairs' lanes
    if (w < CB) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int row = (i >> 2) * 8 + (l >> 5) * 4 + (i & 3);
            dXs[row * DP + w * 32 + (l & 31)] = acc_dx[i];
        }
    }
    lds_barrier();
    if (live) {
        float4* dxs = reinterpret_cast<float4*>(a.w.dxs + b * D);
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int ci = lp + 16 * i;
            const float4 n = *reinterpret_cast<const float4*>(dXs + p * DP + 4 * ci);
            dxs[ci] = make_float4(fmaf(a.lr, n.x, dxp[i].x), fmaf(a.lr, n.y, dxp[i].y), fmaf(a.lr, n.z, dxp[i].z), fmaf(a.lr, n.w, dxp[i].w));
        }
    }
    if (LOSS) {
        __shared__ double sh[kScoreThreads / 64];
        for (int off = 32; off > 0; off >>= 1) loss += __shfl_xor(loss, off, 64);
        if (l == 0) sh[w] = static_cast<double>(loss);
        __syncthreads();
        if (tid == 0) {
            double total = 0.0;
            for (int i = 0; i < kScoreThreads / 64; ++i) total += sh[i];
            if (total != 0.0) atomicAdd(a.loss, total);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// dctx kernel: dC = G^T . Xq.  Workgroup tile 128 negatives x TD columns (TD = 64 or 128), one share
// of the batch (the contraction index) per blockIdx.z.  Both operands are contraction-contiguous in
// memory (GT [N][Bp], XqT [d][Bp]); 64 contraction steps at a time are staged through LDS so that
// the four wavefronts share them (operand traffic, not arithmetic, bounds this product), with the
// next stage travelling into registers meanwhile.  Wavefront w: 64 negatives (w & 1) x TD/2 columns
// (w >> 1).
// ---------------------------------------------------------------------------------------------
struct DctxArgs {
    SharedWs w;
    int32_t N, D;
};

template <int TD>
__global__ __launch_bounds__(256) void dctx_kernel(DctxArgs a)
{
    constexpr int KP = 64 + 8;        // LDS pitch (bf16)
    constexpr int BT = TD / 64;       // column tiles per wavefront
    constexpr int BPT = TD * 8 / 256; // 16-byte pieces of the column operand per thread
    __shared__ uint16_t As[128 * KP];
    __shared__ uint16_t Bs[TD * KP];
    const int tid = threadIdx.x, l = tid & 63, w = tid >> 6;
    const int wr = w & 1, wc = w >> 1;
    const int64_t Bp = a.w.Bp;
    const int kc = static_cast<int>(Bp / kSplit);
    const int64_t kbeg = static_cast<int64_t>(blockIdx.z) * kc;
    const int n0 = blockIdx.x * 128, d0 = blockIdx.y * TD;
    f32x16 acc[2][BT];
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int t = 0; t < BT; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[r][t][i] = 0.0f;

    // piece c: row c / 8, 16-byte column c % 8
    const uint16_t* src_a[4];
    const uint16_t* src_b[BPT];
    u32x4 pa[4], pb[BPT];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = tid + i * 256;
        src_a[i] = a.w.GT + static_cast<int64_t>(n0 + c / 8) * Bp + kbeg + (c % 8) * 8;
        pa[i] = *reinterpret_cast<const u32x4*>(src_a[i]);
    }
#pragma unroll
    for (int i = 0; i < BPT; ++i) {
        const int c = tid + i * 256;
        src_b[i] = a.w.XqT + static_cast<int64_t>(d0 + c / 8) * Bp + kbeg + (c % 8) * 8;
        pb[i] = *reinterpret_cast<const u32x4*>(src_b[i]);
    }
    for (int k0 = 0; k0 < kc; k0 += 64) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c = tid + i * 256;
            *reinterpret_cast<u32x4*>(As + (c / 8) * KP + (c % 8) * 8) = pa[i];
        }
#pragma unroll
        for (int i = 0; i < BPT; ++i) {
            const int c = tid + i * 256;
            *reinterpret_cast<u32x4*>(Bs + (c / 8) * KP + (c % 8) * 8) = pb[i];
        }
        __syncthreads();
        if (k0 + 64 < kc) {
#pragma unroll
            for (int i = 0; i < 4; ++i) { src_a[i] += 64; pa[i] = *reinterpret_cast<const u32x4*>(src_a[i]); }
#pragma unroll
            for (int i = 0; i < BPT; ++i) { src_b[i] += 64; pb[i] = *reinterpret_cast<const u32x4*>(src_b[i]); }
        }
        const uint16_t* ar = As + (wr * 64 + (l & 31)) * KP + (l >> 5) * 8;
        const uint16_t* br = Bs + (wc * (TD / 2) + (l & 31)) * KP + (l >> 5) * 8;
#pragma unroll
        for (int kk = 0; kk < 64; kk += 16) {
            const bf16x8 a0 = as_bf16x8(*reinterpret_cast<const uint4*>(ar + kk));
            const bf16x8 a1 = as_bf16x8(*reinterpret_cast<const uint4*>(ar + 32 * KP + kk));
#pragma unroll
            for (int t = 0; t < BT; ++t) {
                const bf16x8 bv = as_bf16x8(*reinterpret_cast<const uint4*>(br + t * 32 * KP + kk));
                acc[0][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, bv, acc[0][t], 0, 0, 0);
                acc[1][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, bv, acc[1][t], 0, 0, 0);
            }
        }
        __syncthreads();
    }
    float* out = a.w.dCp + static_cast<int64_t>(blockIdx.z) * a.N * a.D;
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int t = 0; t < BT; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int row = n0 + wr * 64 + r * 32 + (i >> 2) * 8 + (l >> 5) * 4 + (i & 3);
                const int col = d0 + wc * (TD / 2) + t * 32 + (l & 31);
                out[static_cast<int64_t>(row) * a.D + col] = acc[r][t][i];
            }
}

// ---------------------------------------------------------------------------------------------
// update kernel: one lane group of G = D/8 lanes per pair / per negative.  Nothing reads the tables
// any more, so every staged delta is simply added to its row.  fp32 atomics retire far more slowly
// than plain stores on this chip, so a row that a single reference of the batch names (it owns its
// key's position and nobody flagged it) is read, added to and stored back in float4 pieces; only
// rows named more than once, and the few whose key lost its position to another row, take atomics
// (lane lg then owns elements lg + m*G, so each atomic instruction covers consecutive dwords).
// ---------------------------------------------------------------------------------------------
struct UpdateArgs {
    float* X;
    float* C;
    const int2* pairs;
    int64_t B;
    int32_t N;
    float lr;
    SharedWs w;
};

__device__ __forceinline__ bool sole_reference(const SharedWs& w, uint32_t key, uint32_t ref)
{
    const uint32_t pos = ref_hash(key, w.hash_mask);
    return w.slots[pos] == ref_entry(key, ref) && w.multi[pos] == 0;
}

__device__ __forceinline__ float4 add4(float4 a, float4 b) { return make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w); }

template <int D>
__global__ __launch_bounds__(256) void update_shared_kernel(UpdateArgs a)
{
    constexpr int G = D / 8;
    constexpr int GROUPS = 256 / G;
    const int lg = threadIdx.x & (G - 1);
    const int64_t gidx = static_cast<int64_t>(blockIdx.x) * GROUPS + threadIdx.x / G;
    if (gidx < a.B) {
        const int2 pr = a.pairs[gidx];
        const bool x_sole = sole_reference(a.w, static_cast<uint32_t>(pr.x), static_cast<uint32_t>(2 * gidx));
        const bool c_sole = sole_reference(a.w, static_cast<uint32_t>(pr.y) | kContextKey, static_cast<uint32_t>(2 * gidx + 1));
        float* xrow = a.X + static_cast<int64_t>(pr.x) * D;
        float* crow = a.C + static_cast<int64_t>(pr.y) * D;
        const float* dxs = a.w.dxs + gidx * D;
        const float* dcs = a.w.dcs + gidx * D;
        // all loads of a group are issued before its first store or atomic
        float4 x4[2], c4[2];
        float x1[8], c1[8];
        if (x_sole) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int ci = lg + i * G;
                x4[i] = add4(reinterpret_cast<const float4*>(xrow)[ci], reinterpret_cast<const float4*>(dxs)[ci]);
            }
        } else {
#pragma unroll
            for (int m = 0; m < 8; ++m) x1[m] = dxs[lg + m * G];
        }
        if (c_sole) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int ci = lg + i * G;
                c4[i] = add4(reinterpret_cast<const float4*>(crow)[ci], reinterpret_cast<const float4*>(dcs)[ci]);
            }
        } else {
#pragma unroll
            for (int m = 0; m < 8; ++m) c1[m] = dcs[lg + m * G];
        }
        if (x_sole) {
#pragma unroll
            for (int i = 0; i < 2; ++i) reinterpret_cast<float4*>(xrow)[lg + i * G] = x4[i];
        } else {
#pragma unroll
            for (int m = 0; m < 8; ++m) unsafeAtomicAdd(xrow + lg + m * G, x1[m]);
        }
        if (c_sole) {
#pragma unroll
            for (int i = 0; i < 2; ++i) reinterpret_cast<float4*>(crow)[lg + i * G] = c4[i];
        } else {
#pragma unroll
            for (int m = 0; m < 8; ++m) unsafeAtomicAdd(crow + lg + m * G, c1[m]);
        }
    } else if (gidx < a.B + a.N) {
        const int64_t j = gidx - a.B;
        const int32_t id = a.w.negids[j];
        const bool sole = sole_reference(a.w, static_cast<uint32_t>(id) | kContextKey, static_cast<uint32_t>(2 * a.B + j));
        float* crow = a.C + static_cast<int64_t>(id) * D;
        if (sole) {
            float4 c4[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int ci = lg + i * G;
                float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                for (int s = 0; s < kSplit; ++s)
                    sum = add4(sum, reinterpret_cast<const float4*>(a.w.dCp + (static_cast<int64_t>(s) * a.N + j) * D)[ci]);
                const float4 r = reinterpret_cast<const float4*>(crow)[ci];
                c4[i] = make_float4(fmaf(a.lr, sum.x, r.x), fmaf(a.lr, sum.y, r.y), fmaf(a.lr, sum.z, r.z), fmaf(a.lr, sum.w, r.w));
            }
#pragma unroll
            for (int i = 0; i < 2; ++i) reinterpret_cast<float4*>(crow)[lg + i * G] = c4[i];
        } else {
            float c1[8];
#pragma unroll
            for (int m = 0; m < 8; ++m) {
                const int e = lg + m * G;
                float sum = 0.0f;
#pragma unroll
                for (int s = 0; s < kSplit; ++s) sum += a.w.dCp[(static_cast<int64_t>(s) * a.N + j) * D + e];
                c1[m] = a.lr * sum;
            }
#pragma unroll
            for (int m = 0; m < 8; ++m) unsafeAtomicAdd(crow + lg + m * G, c1[m]);
        }
    }
}

template <int D>
hipError_t run_shared(ne_tables* t, const ne_alias* al, const int32_t* pairs_dev, int64_t B, int32_t N, float lr,
                      float neg_scale, uint64_t batch_index, const SharedWs& w, int32_t* neg_out, double* loss,
                      hipStream_t st)
{
    constexpr int G = D / 8;
    constexpr int GROUPS = 256 / G;
    PrepNegArgs pa{};
    pa.C = reinterpret_cast<const float4*>(t->context); pa.pairs = reinterpret_cast<const int2*>(pairs_dev);
    pa.B = B; pa.N = N; pa.batch_index = batch_index;
    pa.k0 = static_cast<uint32_t>(t->seed); pa.k1 = static_cast<uint32_t>(t->seed >> 32);
    pa.alias = al->table; pa.alias_n = static_cast<uint64_t>(al->n); pa.alias_base = al->base;
    pa.w = w; pa.neg_out = neg_out;
    // threads: a lane group per negative, one per pair reference, one per 16 flags
    int64_t threads = static_cast<int64_t>(N) * G;
    if (threads < 2 * B) threads = 2 * B;
    if (threads < (static_cast<int64_t>(w.hash_mask) + 16) / 16) threads = (static_cast<int64_t>(w.hash_mask) + 16) / 16;
    hipLaunchKernelGGL(prep_kernel<D>, dim3(static_cast<unsigned>((threads + 255) / 256)), dim3(256), 0, st, pa);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;

    ScoresArgs ca{};
    ca.X = reinterpret_cast<const float4*>(t->vertex); ca.C = pa.C;
    ca.w = w; ca.B = B; ca.N = N; ca.lr = lr; ca.neg_scale = neg_scale; ca.loss = loss; ca.pairs = pa.pairs;
    const bool timed = profile_begin(t, st);
    if (loss)
        hipLaunchKernelGGL((scores_kernel<D, true>), dim3(static_cast<unsigned>(w.Bp / kPairTile)), dim3(kScoreThreads), 0, st, ca);
    else
        hipLaunchKernelGGL((scores_kernel<D, false>), dim3(static_cast<unsigned>(w.Bp / kPairTile)), dim3(kScoreThreads), 0, st, ca);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (timed) profile_end(t, st);
    t->batches_done += 1;

    DctxArgs da{};
    da.w = w; da.N = N; da.D = D;
    if (D >= 128)
        hipLaunchKernelGGL(dctx_kernel<128>, dim3(N / 128, D / 128, kSplit), dim3(256), 0, st, da);
    else
        hipLaunchKernelGGL(dctx_kernel<64>, dim3(N / 128, 1, kSplit), dim3(256), 0, st, da);
    e = hipGetLastError();
    if (e != hipSuccess) return e;

    UpdateArgs ua{};
    ua.X = t->vertex; ua.C = t->context; ua.pairs = pa.pairs; ua.B = B; ua.N = N; ua.lr = lr; ua.w = w;
    hipLaunchKernelGGL(update_shared_kernel<D>, dim3(static_cast<unsigned>((B + N + GROUPS - 1) / GROUPS)), dim3(256), 0, st, ua);
    return hipGetLastError();
}

}  // namespace

extern "C" {

size_t ne_shared_workspace_bytes(int32_t dim, int64_t B, int32_t N)
{
    SharedWs w;
    if (!shared_layout(dim, B, N, nullptr, &w)) return 0;
    return w.total;
}

// Argument checks and launches common to both entry points; `what` names the workspace in messages.
static ne_status train_shared_impl(ne_tables* t, const ne_alias* al, const int32_t* pairs_dev, int64_t B, int32_t N, float lr,
                                   float neg_scale, uint64_t batch_index, void* workspace_dev, size_t workspace_bytes,
                                   bool static_scratch, int32_t* neg_out_dev, double* loss_sum_dev, void* hip_stream)
{
    if (!t || !al) return fail(NE_ERR_ARG, "tables or alias handle is NULL");
    if (B < 0) return fail(NE_ERR_ARG, "B is negative");
    if (B == 0) return NE_OK;
    if (!pairs_dev || !aligned(pairs_dev, 8)) return fail(NE_ERR_ARG, "pairs_dev is NULL or not 8-byte aligned");
    if (!std::isfinite(lr) || !std::isfinite(neg_scale)) return fail(NE_ERR_ARG, "lr or neg_scale is not finite");
    if (al->base < 0 || al->base + al->n > t->num_nodes)
        return fail(NE_ERR_STATE, "alias id range [base, base+n) is not inside the tables' [0, num_nodes)");
    SharedWs w;
    if (!shared_layout(t->dim, B, N, static_cast<char*>(workspace_dev), &w))
        return fail(NE_ERR_ARG, "shared-negative mode needs dim in {64, 128, 256}, 1 <= B <= 2^20, N a multiple of 128 in [128, 65536]");
    if (static_scratch) {
        if (w.total > workspace_bytes)
            return fail(NE_ERR_ARG, "this (dim, B, N) needs " + std::to_string(w.total) + " bytes of scratch; the static scratch of "
                                    "ne_train_batch_shared_static holds " + std::to_string(workspace_bytes) +
                                    " (NE_SHARED_STATIC_SCRATCH_BYTES): use ne_train_batch_shared with a workspace of the caller");
    } else if (!workspace_dev || !aligned(workspace_dev, 256) || workspace_bytes < w.total) {
        return fail(NE_ERR_ARG, "workspace_dev is NULL, not 256-byte aligned, or smaller than ne_shared_workspace_bytes()");
    }
    if (loss_sum_dev && !aligned(loss_sum_dev, 8)) return fail(NE_ERR_ARG, "loss_sum_dev is misaligned");
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    hipError_t e = hipErrorInvalidValue;
    switch (t->dim) {
        case 64: e = run_shared<64>(t, al, pairs_dev, B, N, lr, neg_scale, batch_index, w, neg_out_dev, loss_sum_dev, st); break;
        case 128: e = run_shared<128>(t, al, pairs_dev, B, N, lr, neg_scale, batch_index, w, neg_out_dev, loss_sum_dev, st); break;
        case 256: e = run_shared<256>(t, al, pairs_dev, B, N, lr, neg_scale, batch_index, w, neg_out_dev, loss_sum_dev, st); break;
        default: break;
    }
    if (e != hipSuccess) return fail(NE_ERR_HIP, std::string("shared-negative launch: ") + hipGetErrorString(e));
    return NE_OK;
}

// Device address of `scratch` on the current device, looked up once per device (every GPU holds its
// own copy of the array at its own address).
static ne_status static_scratch_of_current_device(void** out)
{
    constexpr int kMaxDevices = 64;
    static std::mutex lock;
    static void* address[kMaxDevices] = {};
    int device = -1;
    NE_HIP_CHECK(hipGetDevice(&device));
    if (device < 0 || device >= kMaxDevices) return fail(NE_ERR_STATE, "device index outside [0, 64)");
    std::lock_guard<std::mutex> guard(lock);
    if (!address[device]) {
        void* p = nullptr;
        NE_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p || !aligned(p, 256)) return fail(NE_ERR_HIP, "hipGetSymbolAddress returned no usable address for the static scratch");
        address[device] = p;
    }
    *out = address[device];
    return NE_OK;
}

ne_status ne_train_batch_shared(ne_tables* t, const ne_alias* al, const int32_t* pairs_dev, int64_t B, int32_t N,
                                float lr, float neg_scale, uint64_t batch_index, void* workspace_dev,
                                size_t workspace_bytes, int32_t* neg_out_dev, double* loss_sum_dev, void* hip_stream)
{
    return train_shared_impl(t, al, pairs_dev, B, N, lr, neg_scale, batch_index, workspace_dev, workspace_bytes, false,
                             neg_out_dev, loss_sum_dev, hip_stream);
}

ne_status ne_train_batch_shared_static(ne_tables* t, const ne_alias* al, const int32_t* pairs_dev, int64_t B, int32_t N,
                                       float lr, float neg_scale, uint64_t batch_index, int32_t* neg_out_dev,
                                       double* loss_sum_dev, void* hip_stream)
{
    void* ws = nullptr;
    const ne_status rc = static_scratch_of_current_device(&ws);
    if (rc != NE_OK) return rc;
    return train_shared_impl(t, al, pairs_dev, B, N, lr, neg_scale, batch_index, ws, kStaticScratchBytes, true,
                             neg_out_dev, loss_sum_dev, hip_stream);
}

}  // extern "C"
