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
// Four kernels per batch:
//   stage   gathers and rounds the rows, draws the N negatives, does the positive pairs in fp32 and
//           stages their deltas; the tables are only read.
//   scores  one workgroup per 128 pairs and share of the negatives: S tile by tile on MFMA, sigmoid
//           in registers, G to LDS (and transposed to memory for the dC product), dX accumulated on
//           MFMA over the share.
//   dctx    dC = G^T . Xq on MFMA, split over the batch dimension into partial sums.
//   update  adds every staged delta to the tables.  Nothing reads the tables any more at that point,
//           so duplicates simply add up: rows named once in the batch (found with the plain-store
//           claim of the stage kernel and the resolve pass that rides in the scores kernel) are
//           rewritten with plain stores, the others take fp32 atomics.
#include <hip/hip_bf16.h>

#include <atomic>
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

constexpr int kRowTile = 128;    // pairs per workgroup in the scores kernel
constexpr int kScoreThreads = 512;  // 8 wavefronts: two per SIMD, so that one's LDS traffic overlaps the other's MFMAs
constexpr int kNegChunk = 64;    // negatives per LDS chunk in the scores kernel
constexpr int kSplit = 16;       // partial sums of the dC product
constexpr int kNegSplit = 4;     // at most this many workgroups per row tile in the scores kernel, each taking a share of the negatives
constexpr int kBatchPad = 1024;  // the padded batch is a multiple of this (kSplit shares of whole 64-pair steps)

__device__ __forceinline__ uint16_t to_bf16(float x)
{
    uint32_t u = __float_as_uint(x);
    u += 0x7FFFu + ((u >> 16) & 1u);   // round to nearest even
    return static_cast<uint16_t>(u >> 16);
}

// sigmoid from the hardware exp2 and reciprocal (about 1 ulp each): the result is rounded to bf16 anyway
__device__ __forceinline__ float fast_sigmoidf(float z) { return __frcp_rn(1.0f + __expf(-z)); }

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

struct SharedWs {
    uint16_t* Xq;    // [Bp][d]   bf16 source rows (zero beyond B)
    uint16_t* XqT;   // [d][Bp]
    uint16_t* Cq;    // [N][d]    bf16 negative rows
    uint16_t* CqT;   // [d][N]
    uint16_t* GT;    // [N][Bp]   bf16 coefficients, transposed
    float* dxp;      // [Bp][d]   lr * g0 * c_ctx          (positive pair, source side)
    float* uctx;     // [Bp][d]   lr * g0 * x              (positive pair, context side)
    float* dXn;      // [kNegSplit][Bp][d]   partial sums of G . Cq
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
    w->Xq = reinterpret_cast<uint16_t*>(take(Bp * d * 2));
    w->XqT = reinterpret_cast<uint16_t*>(take(Bp * d * 2));
    w->Cq = reinterpret_cast<uint16_t*>(take(n * d * 2));
    w->CqT = reinterpret_cast<uint16_t*>(take(n * d * 2));
    w->GT = reinterpret_cast<uint16_t*>(take(n * Bp * 2));
    w->dxp = reinterpret_cast<float*>(take(Bp * d * 4));
    w->uctx = reinterpret_cast<float*>(take(Bp * d * 4));
    w->dXn = reinterpret_cast<float*>(take(static_cast<size_t>(kNegSplit) * Bp * d * 4));
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
// stage kernel.  One lane group of G = D/8 lanes per row: groups [0, Bp) are the pairs, groups
// [Bp, Bp+N) the negatives.  Lane lg holds the float4 chunks lg and lg+G of its row.
// ---------------------------------------------------------------------------------------------
struct StageArgs {
    const float4* X;
    const float4* C;
    const int2* pairs;
    int64_t B, Bp;
    int32_t N;
    float lr;
    uint64_t batch_index;
    uint32_t k0, k1;
    const uint2* alias;
    uint64_t alias_n;
    int32_t alias_base;
    SharedWs w;
    int32_t* neg_out;
    double* loss;
};

template <int D>
__global__ __launch_bounds__(256) void stage_kernel(StageArgs a)
{
    constexpr int G = D / 8;
    constexpr int GROUPS = 256 / G;
    constexpr int D4 = D / 4;
    const int lg = threadIdx.x & (G - 1);
    const int64_t gidx = static_cast<int64_t>(blockIdx.x) * GROUPS + threadIdx.x / G;
    float loss_term = 0.0f;
    // the "named more than once" flags start from zero in every batch (16 per thread; the grid has
    // more than (2 Bp + N) * 8 threads and the flag array 4..8 times (2 Bp + N) bytes)
    {
        const size_t i = (static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x) * 16;
        if (i <= a.w.hash_mask) *reinterpret_cast<uint4*>(a.w.multi + i) = make_uint4(0u, 0u, 0u, 0u);
    }
    if (gidx < a.Bp) {
        const int64_t b = gidx;
        uint2* xq = reinterpret_cast<uint2*>(a.w.Xq + b * D);
        if (b < a.B) {
            const int2 pr = a.pairs[b];
            // claim: whichever reference stores last owns the position of its row's key
            if (lg < 2) {
                const uint32_t key = lg == 0 ? static_cast<uint32_t>(pr.x) : (static_cast<uint32_t>(pr.y) | kContextKey);
                a.w.slots[ref_hash(key, a.w.hash_mask)] = ref_entry(key, static_cast<uint32_t>(2 * b + lg));
            }
            const float4* xrow = a.X + static_cast<int64_t>(pr.x) * D4;
            const float4* crow = a.C + static_cast<int64_t>(pr.y) * D4;
            float4 x[2], c[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) { x[i] = xrow[lg + i * G]; c[i] = crow[lg + i * G]; }
            const float s0 = group_sum<G>(dot4(x[0], c[0]) + dot4(x[1], c[1]));
            const float g0 = a.lr * (1.0f - sigmoidf(s0));
            if (lg == 0) loss_term = softplusf(-s0);
            float4* dxp = reinterpret_cast<float4*>(a.w.dxp + b * D);
            float4* uctx = reinterpret_cast<float4*>(a.w.uctx + b * D);
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int ci = lg + i * G;
                dxp[ci] = make_float4(g0 * c[i].x, g0 * c[i].y, g0 * c[i].z, g0 * c[i].w);
                uctx[ci] = make_float4(g0 * x[i].x, g0 * x[i].y, g0 * x[i].z, g0 * x[i].w);
                xq[ci] = make_uint2(to_bf16(x[i].x) | (static_cast<uint32_t>(to_bf16(x[i].y)) << 16),
                                    to_bf16(x[i].z) | (static_cast<uint32_t>(to_bf16(x[i].w)) << 16));
            }
        } else {
#pragma unroll
            for (int i = 0; i < 2; ++i) xq[lg + i * G] = make_uint2(0u, 0u);   // padding rows score zero
        }
    } else if (gidx < a.Bp + a.N) {
        const int32_t j = static_cast<int32_t>(gidx - a.Bp);
        const uint4 r = philox4x32_10(make_uint4(static_cast<uint32_t>(a.batch_index), static_cast<uint32_t>(a.batch_index >> 32),
                                                 static_cast<uint32_t>(j), kStreamSharedNegative), a.k0, a.k1);
        const int32_t id = a.alias_base + alias_draw(r, a.alias, a.alias_n);
        if (lg == 0) {
            a.w.negids[j] = id;
            if (a.neg_out) a.neg_out[j] = id;
            const uint32_t key = static_cast<uint32_t>(id) | kContextKey;
            a.w.slots[ref_hash(key, a.w.hash_mask)] = ref_entry(key, static_cast<uint32_t>(2 * a.B + j));
        }
        const float4* crow = a.C + static_cast<int64_t>(id) * D4;
        uint2* cq = reinterpret_cast<uint2*>(a.w.Cq + static_cast<int64_t>(j) * D);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int ci = lg + i * G;
            const float4 c = crow[ci];
            const uint16_t h0 = to_bf16(c.x), h1 = to_bf16(c.y), h2 = to_bf16(c.z), h3 = to_bf16(c.w);
            cq[ci] = make_uint2(h0 | (static_cast<uint32_t>(h1) << 16), h2 | (static_cast<uint32_t>(h3) << 16));
            uint16_t* ct = a.w.CqT + static_cast<int64_t>(4 * ci) * a.N + j;
            ct[0] = h0; ct[a.N] = h1; ct[2 * static_cast<int64_t>(a.N)] = h2; ct[3 * static_cast<int64_t>(a.N)] = h3;
        }
    }
    if (a.loss) {   // uniform over the grid
        __shared__ double sh[4];
        float l = loss_term;
        for (int off = 32; off > 0; off >>= 1) l += __shfl_xor(l, off, 64);
        if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = static_cast<double>(l);
        __syncthreads();
        if (threadIdx.x == 0) {
            const double t = sh[0] + sh[1] + sh[2] + sh[3];
            if (t != 0.0) atomicAdd(a.loss, t);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// scores kernel: one workgroup (8 wavefronts) per 128 pairs and share of the negatives.
//   wavefront w: row quarter rh = w & 3 (32 pairs); column half ch = w >> 2
//   S tile   : pairs rh*32.. x negatives ch*32.. of the current 64-negative chunk   (1 MFMA tile)
//   dX tiles : pairs rh*32.. x columns ch*D/2 .. ch*D/2 + D/2                        (D/64 tiles)
// MFMA 32x32x16 operand layout (checked on hardware): lane l supplies row/column l%32 and the 8
// consecutive k values (l/32)*8..+7; accumulator element i is row (i/4)*8 + (l/32)*4 + i%4, column l%32.
// LDS rows are padded by 8 bf16 so that the 16-byte fragment reads of 32 rows spread over all banks.
// ---------------------------------------------------------------------------------------------
struct ScoresArgs {
    SharedWs w;
    int64_t B;
    int32_t N;
    float neg_scale;
    double* loss;
    const int2* pairs;
};

// Column of G inside its LDS row: the eight 16-byte groups of a row are permuted by the row's 16-row
// block, so that the transposed read-out below (one negative, rows 16 apart) spreads over the banks
// while a fragment read (one row, 8 consecutive negatives) stays one 16-byte access.
__device__ __forceinline__ int g_col(int row, int col) { return ((((col >> 3) ^ (row >> 4)) & 7) << 3) | (col & 7); }

template <int D>
__global__ __launch_bounds__(kScoreThreads) void scores_kernel(ScoresArgs a)
{
    constexpr int XP = D + 8;            // pitch of Xs and Cs rows (bf16)
    constexpr int TP = kNegChunk + 8;    // pitch of CTs and Gs rows
    constexpr int DT = D / 64;           // dX tiles per wavefront
    extern __shared__ uint16_t lds[];
    uint16_t* Xs = lds;                              // [128][XP]
    uint16_t* Cs = Xs + kRowTile * XP;               // [64][XP]
    uint16_t* CTs = Cs + kNegChunk * XP;             // [D][TP]
    uint16_t* Gs = CTs + D * TP;                     // [128][TP]
    const int tid = threadIdx.x;
    const int l = tid & 63, w = tid >> 6;
    const int rh = w & 3, ch = w >> 2;   // 32-pair quarter, half of the chunk / of the columns
    const int64_t b0 = static_cast<int64_t>(blockIdx.x) * kRowTile;
    const int64_t Bp = a.w.Bp;

    // resolve (ids only, a by-product of this launch): a reference that finds its row's key at the
    // key's position under another reference's name flags the row as named more than once
    {
        const int64_t refs = 2 * a.B + a.N;
        const int64_t stride = static_cast<int64_t>(gridDim.x) * gridDim.y * kScoreThreads;
        for (int64_t r = (static_cast<int64_t>(blockIdx.y) * gridDim.x + blockIdx.x) * kScoreThreads + tid; r < refs; r += stride) {
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

    // the source rows of this workgroup
    for (int c = tid; c < kRowTile * (D / 8); c += kScoreThreads) {
        const int r = c / (D / 8), q = c % (D / 8);
        *reinterpret_cast<uint4*>(Xs + r * XP + q * 8) = *reinterpret_cast<const uint4*>(a.w.Xq + (b0 + r) * D + q * 8);
    }
    __syncthreads();
    // by-product: the transposed copy the dC product reads
    for (int col = tid; col < D && blockIdx.y == 0; col += kScoreThreads) {
        uint16_t* out = a.w.XqT + static_cast<int64_t>(col) * Bp + b0;
#pragma unroll
        for (int r0 = 0; r0 < kRowTile; r0 += 8) {
            uint32_t p[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                p[i] = Xs[(r0 + 2 * i) * XP + col] | (static_cast<uint32_t>(Xs[(r0 + 2 * i + 1) * XP + col]) << 16);
            *reinterpret_cast<uint4*>(out + r0) = make_uint4(p[0], p[1], p[2], p[3]);
        }
    }

    f32x16 acc_dx[DT];
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc_dx[t][i] = 0.0f;
    float loss = 0.0f;

    // this workgroup's share of the negatives, in chunks of 64; the next chunk's rows travel from
    // memory into registers while the current one is being used
    constexpr int CPT = kNegChunk * (D / 8) / kScoreThreads;   // 16-byte pieces of Cs per thread (= of CTs)
    const int n_share = a.N / static_cast<int>(gridDim.y);
    const int n_begin = blockIdx.y * n_share, n_end = n_begin + n_share;
    u32x4 pc[CPT], pt[CPT];
    // piece c of the chunk: Cs row c / (D/8), 16-byte column c % (D/8); CTs row c / 8, column c % 8
    const uint16_t* src_c[CPT];
    const uint16_t* src_t[CPT];
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
        const int c = tid + i * kScoreThreads;
        src_c[i] = a.w.Cq + static_cast<int64_t>(n_begin + c / (D / 8)) * D + (c % (D / 8)) * 8;
        src_t[i] = a.w.CqT + static_cast<int64_t>(c / (kNegChunk / 8)) * a.N + n_begin + (c % (kNegChunk / 8)) * 8;
        pc[i] = *reinterpret_cast<const u32x4*>(src_c[i]);
        pt[i] = *reinterpret_cast<const u32x4*>(src_t[i]);
    }
    for (int n0 = n_begin; n0 < n_end; n0 += kNegChunk) {
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            const int c = tid + i * kScoreThreads;
            *reinterpret_cast<u32x4*>(Cs + (c / (D / 8)) * XP + (c % (D / 8)) * 8) = pc[i];
            *reinterpret_cast<u32x4*>(CTs + (c / (kNegChunk / 8)) * TP + (c % (kNegChunk / 8)) * 8) = pt[i];
        }
        __syncthreads();
        if (n0 + kNegChunk < n_end) {
#pragma unroll
            for (int i = 0; i < CPT; ++i) {
                src_c[i] += kNegChunk * D;
                src_t[i] += kNegChunk;
                pc[i] = *reinterpret_cast<const u32x4*>(src_c[i]);
                pt[i] = *reinterpret_cast<const u32x4*>(src_t[i]);
            }
        }

        // S = Xq . Cq^T for 32 pairs x 32 negatives
        f32x16 s;
#pragma unroll
        for (int i = 0; i < 16; ++i) s[i] = 0.0f;
        const uint16_t* xa = Xs + (rh * 32 + (l & 31)) * XP + (l >> 5) * 8;
        const uint16_t* cb = Cs + (ch * 32 + (l & 31)) * XP + (l >> 5) * 8;
#pragma unroll
        for (int k0 = 0; k0 < D; k0 += 16) {
            const bf16x8 av = as_bf16x8(*reinterpret_cast<const uint4*>(xa + k0));
            const bf16x8 bv = as_bf16x8(*reinterpret_cast<const uint4*>(cb + k0));
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, s, 0, 0, 0);
        }
        // G = -neg_scale * sigmoid(S), zero for padding rows; into LDS as bf16
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int row = rh * 32 + (i >> 2) * 8 + (l >> 5) * 4 + (i & 3);
            const int col = ch * 32 + (l & 31);
            const bool valid = b0 + row < a.B;
            const float g = valid ? -a.neg_scale * fast_sigmoidf(s[i]) : 0.0f;
            if (a.loss && valid) loss += a.neg_scale * softplusf(s[i]);
            Gs[row * TP + g_col(row, col)] = to_bf16(g);
        }
        __syncthreads();

        // G^T to memory: 64 negatives x 128 pairs, 256 contiguous bytes per negative
        {
            const int neg = tid >> 3, part = tid & 7;
            uint32_t p[8];
#pragma unroll
            for (int i = 0; i < 8; ++i)
                p[i] = Gs[(part * 16 + 2 * i) * TP + g_col(part * 16, neg)] |
                       (static_cast<uint32_t>(Gs[(part * 16 + 2 * i + 1) * TP + g_col(part * 16, neg)]) << 16);
            uint4* out = reinterpret_cast<uint4*>(a.w.GT + static_cast<int64_t>(n0 + neg) * Bp + b0 + part * 16);
            out[0] = make_uint4(p[0], p[1], p[2], p[3]);
            out[1] = make_uint4(p[4], p[5], p[6], p[7]);
        }
        // dX += G . Cq for 32 pairs x D/2 columns over the 64 negatives of the chunk
        const uint16_t* ga = Gs + (rh * 32 + (l & 31)) * TP;
#pragma unroll
        for (int kk = 0; kk < kNegChunk; kk += 16) {
            const bf16x8 av = as_bf16x8(*reinterpret_cast<const uint4*>(ga + g_col(rh * 32 + (l & 31), kk + (l >> 5) * 8)));
#pragma unroll
            for (int t = 0; t < DT; ++t) {
                const uint16_t* tb = CTs + (ch * (D / 2) + t * 32 + (l & 31)) * TP + (l >> 5) * 8 + kk;
                acc_dx[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, as_bf16x8(*reinterpret_cast<const uint4*>(tb)),
                                                                    acc_dx[t], 0, 0, 0);
            }
        }
        __syncthreads();   // Cs, CTs, Gs are rewritten by the next chunk
    }

    float* dxn = a.w.dXn + static_cast<int64_t>(blockIdx.y) * Bp * D;
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int row = rh * 32 + (i >> 2) * 8 + (l >> 5) * 4 + (i & 3);
            const int col = ch * (D / 2) + t * 32 + (l & 31);
            dxn[(b0 + row) * D + col] = acc_dx[t][i];
        }
    if (a.loss) {
        __shared__ double sh[kScoreThreads / 64];
        for (int off = 32; off > 0; off >>= 1) loss += __shfl_xor(loss, off, 64);
        if (l == 0) sh[w] = static_cast<double>(loss);
        __syncthreads();
        if (tid == 0) {
            double total = 0.0;
            for (int i = 0; i < kScoreThreads / 64; ++i) total += sh[i];
            atomicAdd(a.loss, total);
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
    int32_t neg_split;   // partial sums of dXn that were written
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
        const float* dxp = a.w.dxp + gidx * D;
        const float* dxn = a.w.dXn + gidx * D;
        const int64_t part = a.w.Bp * D;
        const float* uctx = a.w.uctx + gidx * D;
        // all loads of a group are issued before its first store or atomic
        float4 x4[2], c4[2];
        float x1[8], c1[8];
        if (x_sole) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int ci = lg + i * G;
                float4 n = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                for (int s = 0; s < kNegSplit; ++s)
                    if (s < a.neg_split) n = add4(n, reinterpret_cast<const float4*>(dxn + s * part)[ci]);
                const float4 p = reinterpret_cast<const float4*>(dxp)[ci];
                const float4 r = reinterpret_cast<const float4*>(xrow)[ci];
                x4[i] = make_float4(r.x + fmaf(a.lr, n.x, p.x), r.y + fmaf(a.lr, n.y, p.y), r.z + fmaf(a.lr, n.z, p.z),
                                    r.w + fmaf(a.lr, n.w, p.w));
            }
        } else {
#pragma unroll
            for (int m = 0; m < 8; ++m) {
                const int e = lg + m * G;
                float n = 0.0f;
#pragma unroll
                for (int s = 0; s < kNegSplit; ++s)
                    if (s < a.neg_split) n += dxn[s * part + e];
                x1[m] = fmaf(a.lr, n, dxp[e]);
            }
        }
        if (c_sole) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int ci = lg + i * G;
                c4[i] = add4(reinterpret_cast<const float4*>(crow)[ci], reinterpret_cast<const float4*>(uctx)[ci]);
            }
        } else {
#pragma unroll
            for (int m = 0; m < 8; ++m) c1[m] = uctx[lg + m * G];
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
    StageArgs sa{};
    sa.X = reinterpret_cast<const float4*>(t->vertex); sa.C = reinterpret_cast<const float4*>(t->context);
    sa.pairs = reinterpret_cast<const int2*>(pairs_dev); sa.B = B; sa.Bp = w.Bp; sa.N = N; sa.lr = lr;
    sa.batch_index = batch_index; sa.k0 = static_cast<uint32_t>(t->seed); sa.k1 = static_cast<uint32_t>(t->seed >> 32);
    sa.alias = al->table; sa.alias_n = static_cast<uint64_t>(al->n); sa.alias_base = al->base;
    sa.w = w; sa.neg_out = neg_out; sa.loss = loss;
    hipLaunchKernelGGL(stage_kernel<D>, dim3(static_cast<unsigned>((w.Bp + N + GROUPS - 1) / GROUPS)), dim3(256), 0, st, sa);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;

    // shares of the negatives must be whole 64-negative chunks
    const unsigned neg_split = (N % (kNegSplit * kNegChunk) == 0) ? kNegSplit : 2;
    ScoresArgs ca{};
    ca.w = w; ca.B = B; ca.N = N; ca.neg_scale = neg_scale; ca.loss = loss; ca.pairs = sa.pairs;
    const size_t lds_bytes = (static_cast<size_t>(kRowTile + kNegChunk) * (D + 8) + static_cast<size_t>(D + kRowTile) * (kNegChunk + 8)) * 2;
    // more than the default 64 KB of dynamic LDS (gfx950 has 160 KB per CU): asked for once per device
    // and kernel, so that later calls are kernel launches only (a caller may be capturing the stream)
    {
        static std::atomic<uint64_t> lds_raised{0};
        int device = 0;
        e = hipGetDevice(&device);
        if (e != hipSuccess) return e;
        const uint64_t bit = 1ull << (device & 63);
        if (!(lds_raised.load(std::memory_order_acquire) & bit)) {
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(scores_kernel<D>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    static_cast<int>((static_cast<size_t>(kRowTile + kNegChunk) * (D + 8) +
                                                      static_cast<size_t>(D + kRowTile) * (kNegChunk + 8)) * 2));
            if (e != hipSuccess) return e;
            lds_raised.fetch_or(bit, std::memory_order_release);
        }
    }
    const bool timed = profile_begin(t, st);
    hipLaunchKernelGGL(scores_kernel<D>, dim3(static_cast<unsigned>(w.Bp / kRowTile), neg_split), dim3(kScoreThreads), lds_bytes, st, ca);
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
    ua.X = t->vertex; ua.C = t->context; ua.pairs = sa.pairs; ua.B = B; ua.N = N; ua.lr = lr; ua.neg_split = static_cast<int32_t>(neg_split); ua.w = w;
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
