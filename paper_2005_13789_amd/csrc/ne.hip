// SGNS node-embedding training for MI355X (gfx950): HIP kernels and the C ABI declared in ne.h.
//
// Kernel plan for one batch (Algorithm 1, embedding-training loop; Sec. II-A "Training Process"):
//   score  : one lane group per (src, ctx) pair.  Draws the K negatives (Philox + alias table),
//            gathers x = vertex[src] and the K+1 context rows with dwordx4 loads, reduces the K+1 dot
//            products across the group with DPP, forms g_j and dx = lr * sum_j g_j c_j.  Tables are
//            read-only here.  x, dx, lr*g_j and the ids go to a staging buffer.
//   update : one lane group per pair.  Reads the staged x, dx, g, ids and scatter-adds
//            vertex[src] += dx and context[id_j] += (lr g_j) x with hardware fp32 atomics.
// The kernel boundary between the two is what makes the step minibatch-synchronous: no table row is
// written before every read of the batch has completed.
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
// host-side error plumbing
// ---------------------------------------------------------------------------------------------
static thread_local std::string g_last_error;

static ne_status fail(ne_status st, const std::string& msg)
{
    g_last_error = msg;
    return st;
}

#define NE_HIP_CHECK(expr)                                                                       \
    do {                                                                                         \
        hipError_t e_ = (expr);                                                                  \
        if (e_ != hipSuccess)                                                                    \
            return fail(NE_ERR_HIP, std::string(#expr) + ": " + hipGetErrorString(e_));          \
    } while (0)

struct ne_tables {
    int64_t num_nodes;
    int32_t dim;
    float* vertex;
    float* context;
    uint64_t seed;
};

struct ne_alias {
    const uint2* table;  // device {threshold, alias}[n]
    int64_t n;
    int32_t base;
};

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

// ---------------------------------------------------------------------------------------------
// table initialisation: vertex ~ U(-0.5/d, 0.5/d), context = 0.  One float4 per thread-iteration.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void init_tables_kernel(float4* __restrict__ X, float4* __restrict__ C,
                                                          int64_t num_nodes, int32_t d4, float dimf,
                                                          uint32_t k0, uint32_t k1)
{
    const int64_t total = num_nodes * d4;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < total; i += stride) {
        const uint64_t row = static_cast<uint64_t>(i / d4);
        const uint32_t q = static_cast<uint32_t>(i - static_cast<int64_t>(row) * d4);
        const uint4 r = philox4x32_10(make_uint4(static_cast<uint32_t>(row), static_cast<uint32_t>(row >> 32), q,
                                                 kStreamInit), k0, k1);
        float4 v;
        v.x = ((static_cast<float>(r.x >> 9) + 0.5f) * 0x1p-23f - 0.5f) / dimf;
        v.y = ((static_cast<float>(r.y >> 9) + 0.5f) * 0x1p-23f - 0.5f) / dimf;
        v.z = ((static_cast<float>(r.z >> 9) + 0.5f) * 0x1p-23f - 0.5f) / dimf;
        v.w = ((static_cast<float>(r.w >> 9) + 0.5f) * 0x1p-23f - 0.5f) / dimf;
        X[i] = v;
        C[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
}

// ---------------------------------------------------------------------------------------------
// score kernel.  G lanes per pair, NCH float4 chunks per lane (chunk index = lg + i*G, valid while
// < d4), JB context rows in flight at a time.  TRAIN: writes staging.  !TRAIN: accumulates the loss.
// ---------------------------------------------------------------------------------------------
struct ScoreArgs {
    const float4* X;
    const float4* C;
    const int2* pairs;
    int64_t B;
    int32_t K;
    int32_t d4;
    float lr;
    uint64_t sample_base;
    uint32_t k0, k1;
    const uint2* alias;
    uint64_t alias_n;
    int32_t alias_base;
    float* gbuf;      // [B][K+1]  lr * g_j
    int32_t* nbuf;    // [B][K]    negative ids
    float4* xbuf;     // [B][d4]   copy of x
    float4* dxbuf;    // [B][d4]   lr * sum_j g_j c_j
    int32_t* neg_out; // optional [B][K]
    double* loss;     // eval only
};

template <int G, int NCH, int JB, bool TRAIN>
__global__ __launch_bounds__(256) void score_kernel(ScoreArgs a)
{
    constexpr int GROUPS = 256 / G;
    const int lg = threadIdx.x & (G - 1);
    const int64_t b_raw = static_cast<int64_t>(blockIdx.x) * GROUPS + (threadIdx.x / G);
    const bool active = b_raw < a.B;
    const int64_t b = active ? b_raw : a.B - 1;
    const int K = a.K;
    const int d4 = a.d4;

    const int2 pr = a.pairs[b];

    // lane lg owns row j = lg of the pair: j = 0 the positive context, j = 1..K negative j-1
    int32_t id_mine = pr.y;
    if (lg >= 1 && lg <= K) {
        const uint64_t idx = a.sample_base + static_cast<uint64_t>(b);
        const uint4 r = philox4x32_10(make_uint4(static_cast<uint32_t>(idx), static_cast<uint32_t>(idx >> 32),
                                                 static_cast<uint32_t>(lg - 1), kStreamNegative), a.k0, a.k1);
        id_mine = a.alias_base + alias_draw(r, a.alias, a.alias_n);
        if (active) {
            if (TRAIN) a.nbuf[b * K + (lg - 1)] = id_mine;
            if (a.neg_out) a.neg_out[b * K + (lg - 1)] = id_mine;
        }
    }

    float4 xr[NCH];
    const float4* xrow = a.X + static_cast<int64_t>(pr.x) * d4;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int ci = lg + i * G;
        xr[i] = (ci < d4) ? xrow[ci] : make_float4(0.f, 0.f, 0.f, 0.f);
    }

    float4 dx[NCH];
#pragma unroll
    for (int i = 0; i < NCH; ++i) dx[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    float g_mine = 0.0f;   // lane lg keeps lr*g_lg (TRAIN) or its loss term (eval)

    for (int j0 = 0; j0 <= K; j0 += JB) {
        float4 cr[JB][NCH];
        float part[JB];
#pragma unroll
        for (int jj = 0; jj < JB; ++jj) {
            const int j = j0 + jj;
            const int32_t id = __shfl(id_mine, j <= K ? j : K, G);
            const float4* crow = a.C + static_cast<int64_t>(id) * d4;
#pragma unroll
            for (int i = 0; i < NCH; ++i) {
                const int ci = lg + i * G;
                cr[jj][i] = (j <= K && ci < d4) ? crow[ci] : make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
#pragma unroll
        for (int jj = 0; jj < JB; ++jj) {
            float p = 0.0f;
#pragma unroll
            for (int i = 0; i < NCH; ++i) p += dot4(xr[i], cr[jj][i]);
            part[jj] = p;
        }
#pragma unroll
        for (int jj = 0; jj < JB; ++jj) part[jj] = group_sum<G>(part[jj]);
#pragma unroll
        for (int jj = 0; jj < JB; ++jj) {
            const int j = j0 + jj;
            if (j <= K) {
                const float s = part[jj];
                if (TRAIN) {
                    const float sg = sigmoidf(s);
                    const float g = a.lr * (j == 0 ? 1.0f - sg : -sg);
#pragma unroll
                    for (int i = 0; i < NCH; ++i) {
                        dx[i].x = fmaf(g, cr[jj][i].x, dx[i].x);
                        dx[i].y = fmaf(g, cr[jj][i].y, dx[i].y);
                        dx[i].z = fmaf(g, cr[jj][i].z, dx[i].z);
                        dx[i].w = fmaf(g, cr[jj][i].w, dx[i].w);
                    }
                    if (lg == j) g_mine = g;
                } else {
                    if (lg == j) g_mine = softplusf(j == 0 ? -s : s);
                }
            }
        }
    }

    if (TRAIN) {
        if (active) {
            if (lg <= K) a.gbuf[b * (K + 1) + lg] = g_mine;
            float4* xo = a.xbuf + b * d4;
            float4* dxo = a.dxbuf + b * d4;
#pragma unroll
            for (int i = 0; i < NCH; ++i) {
                const int ci = lg + i * G;
                if (ci < d4) {
                    xo[ci] = xr[i];
                    dxo[ci] = dx[i];
                }
            }
        }
    } else {
        // per-pair loss = sum of the K+1 terms held by lanes 0..K; then block sum in fp64
        float l = (active && lg <= K) ? g_mine : 0.0f;
        l = group_sum<G>(l);
        __shared__ double sh[GROUPS];
        if (lg == 0) sh[threadIdx.x / G] = static_cast<double>(l);
        __syncthreads();
        if (threadIdx.x == 0) {
            double t = 0.0;
            for (int i = 0; i < GROUPS; ++i) t += sh[i];
            atomicAdd(a.loss, t);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// update kernel: scatter-add of the staged deltas with hardware fp32 atomics.
// ---------------------------------------------------------------------------------------------
struct UpdateArgs {
    float* X;
    float* C;
    const int2* pairs;
    int64_t B;
    int32_t K;
    int32_t d4;
    const float* gbuf;
    const int32_t* nbuf;
    const float4* xbuf;
    const float4* dxbuf;
};

__device__ __forceinline__ void atomic_add4(float* p, float4 v)
{
    unsafeAtomicAdd(p + 0, v.x);
    unsafeAtomicAdd(p + 1, v.y);
    unsafeAtomicAdd(p + 2, v.z);
    unsafeAtomicAdd(p + 3, v.w);
}

template <int G, int NCH>
__global__ __launch_bounds__(256) void update_kernel(UpdateArgs a)
{
    constexpr int GROUPS = 256 / G;
    const int lg = threadIdx.x & (G - 1);
    const int64_t b = static_cast<int64_t>(blockIdx.x) * GROUPS + (threadIdx.x / G);
    if (b >= a.B) return;   // whole groups leave together; no cross-group communication below
    const int K = a.K;
    const int d4 = a.d4;
    const int2 pr = a.pairs[b];

    int32_t id_mine = pr.y;
    float g_mine = 0.0f;
    if (lg <= K) {
        g_mine = a.gbuf[b * (K + 1) + lg];
        if (lg >= 1) id_mine = a.nbuf[b * K + (lg - 1)];
    }
    float4 xr[NCH], dx[NCH];
    const float4* xi = a.xbuf + b * d4;
    const float4* dxi = a.dxbuf + b * d4;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int ci = lg + i * G;
        if (ci < d4) {
            xr[i] = xi[ci];
            dx[i] = dxi[ci];
        }
    }
    float* xrow = a.X + static_cast<int64_t>(pr.x) * d4 * 4;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int ci = lg + i * G;
        if (ci < d4) atomic_add4(xrow + 4 * ci, dx[i]);
    }
    for (int j = 0; j <= K; ++j) {
        const int32_t id = __shfl(id_mine, j, G);
        const float g = __shfl(g_mine, j, G);
        float* crow = a.C + static_cast<int64_t>(id) * d4 * 4;
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int ci = lg + i * G;
            if (ci < d4)
                atomic_add4(crow + 4 * ci, make_float4(g * xr[i].x, g * xr[i].y, g * xr[i].z, g * xr[i].w));
        }
    }
}

__global__ __launch_bounds__(256) void validate_pairs_kernel(const int32_t* __restrict__ ids, int64_t count,
                                                             int64_t num_nodes, unsigned long long* bad)
{
    const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
    unsigned long long local = 0;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < count; i += stride) {
        const int32_t v = ids[i];
        local += (v < 0 || v >= num_nodes) ? 1ull : 0ull;
    }
    if (local) atomicAdd(bad, local);
}

// ---------------------------------------------------------------------------------------------
// launch-shape selection
// ---------------------------------------------------------------------------------------------
struct Shape { int G, NCH; };

// Smallest lane group that covers dim/4 float4 chunks and has a lane for each of the K+1 rows.
bool pick_shape(int32_t d4, int32_t K, Shape* out)
{
    static const Shape order[] = {{8, 1}, {16, 1}, {16, 2}, {32, 1}, {32, 2}, {64, 1}, {64, 2}, {64, 4}};
    for (const Shape& s : order) {
        if (s.G * s.NCH >= d4 && s.G >= K + 1) { *out = s; return true; }
    }
    return false;
}

struct StagingLayout { size_t g_off, n_off, x_off, dx_off, total; };

StagingLayout staging_layout(int64_t B, int32_t dim, int32_t K)
{
    auto up = [](size_t v) { return (v + 255) & ~static_cast<size_t>(255); };
    StagingLayout L;
    size_t off = 0;
    L.g_off = off;  off = up(off + static_cast<size_t>(B) * (K + 1) * sizeof(float));
    L.n_off = off;  off = up(off + static_cast<size_t>(B) * (K > 0 ? K : 1) * sizeof(int32_t));
    L.x_off = off;  off = up(off + static_cast<size_t>(B) * dim * sizeof(float));
    L.dx_off = off; off = up(off + static_cast<size_t>(B) * dim * sizeof(float));
    L.total = off;
    return L;
}

template <bool TRAIN>
hipError_t launch_score(const Shape& s, const ScoreArgs& a, hipStream_t st)
{
    const int groups = 256 / s.G;
    const unsigned grid = static_cast<unsigned>((a.B + groups - 1) / groups);
#define NE_SCORE_CASE(G_, N_)                                                                    \
    if (s.G == G_ && s.NCH == N_) {                                                              \
        hipLaunchKernelGGL((score_kernel<G_, N_, 6, TRAIN>), dim3(grid), dim3(256), 0, st, a);   \
        return hipGetLastError();                                                                \
    }
    NE_SCORE_CASE(8, 1) NE_SCORE_CASE(16, 1) NE_SCORE_CASE(16, 2) NE_SCORE_CASE(32, 1)
    NE_SCORE_CASE(32, 2) NE_SCORE_CASE(64, 1) NE_SCORE_CASE(64, 2) NE_SCORE_CASE(64, 4)
#undef NE_SCORE_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_update(const Shape& s, const UpdateArgs& a, hipStream_t st)
{
    const int groups = 256 / s.G;
    const unsigned grid = static_cast<unsigned>((a.B + groups - 1) / groups);
#define NE_UPDATE_CASE(G_, N_)                                                                   \
    if (s.G == G_ && s.NCH == N_) {                                                              \
        hipLaunchKernelGGL((update_kernel<G_, N_>), dim3(grid), dim3(256), 0, st, a);            \
        return hipGetLastError();                                                                \
    }
    NE_UPDATE_CASE(8, 1) NE_UPDATE_CASE(16, 1) NE_UPDATE_CASE(16, 2) NE_UPDATE_CASE(32, 1)
    NE_UPDATE_CASE(32, 2) NE_UPDATE_CASE(64, 1) NE_UPDATE_CASE(64, 2) NE_UPDATE_CASE(64, 4)
#undef NE_UPDATE_CASE
    return hipErrorInvalidValue;
}

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// Largest grid for one launch: batches beyond this many pairs are rejected.
constexpr int64_t kMaxBatch = static_cast<int64_t>(1) << 28;

ne_status check_batch_args(const ne_tables* t, const ne_alias* al, const int32_t* pairs, int64_t B, int32_t K,
                           Shape* shape)
{
    if (!t) return fail(NE_ERR_ARG, "tables handle is NULL");
    if (B < 0 || B > kMaxBatch) return fail(NE_ERR_ARG, "B out of range [0, 2^28]");
    if (K < 0 || K > NE_MAX_NEGATIVES) return fail(NE_ERR_ARG, "K out of range [0, 63]");
    if (K > 0 && !al) return fail(NE_ERR_ARG, "alias handle is NULL but K > 0");
    if (B > 0 && !pairs) return fail(NE_ERR_ARG, "pairs_dev is NULL");
    if (!aligned(pairs, 8)) return fail(NE_ERR_ARG, "pairs_dev must be 8-byte aligned");
    if (al && (al->base < 0 || al->base + al->n > t->num_nodes))
        return fail(NE_ERR_STATE, "alias id range [base, base+n) is not inside the tables' [0, num_nodes)");
    if (!pick_shape(t->dim / 4, K, shape)) return fail(NE_ERR_ARG, "no launch shape for this (dim, K)");
    return NE_OK;
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// C ABI
// ---------------------------------------------------------------------------------------------
extern "C" {

const char* ne_last_error(void) { return g_last_error.c_str(); }

ne_status ne_create_tables(ne_tables** out, int64_t num_nodes, int32_t dim, float* vertex_dev,
                           float* context_dev, uint64_t seed, int32_t init, void* hip_stream)
{
    if (!out) return fail(NE_ERR_ARG, "out is NULL");
    *out = nullptr;
    if (num_nodes <= 0 || num_nodes >= (static_cast<int64_t>(1) << 31))
        return fail(NE_ERR_ARG, "num_nodes must be in (0, 2^31)");
    if (dim < 4 || dim > NE_MAX_DIM || dim % 4 != 0)
        return fail(NE_ERR_ARG, "dim must be a multiple of 4 in [4, 1024]");
    if (!vertex_dev || !context_dev) return fail(NE_ERR_ARG, "table pointer is NULL");
    if (!aligned(vertex_dev, 16) || !aligned(context_dev, 16))
        return fail(NE_ERR_ARG, "table pointers must be 16-byte aligned");
    ne_tables* t = new (std::nothrow) ne_tables{num_nodes, dim, vertex_dev, context_dev, seed};
    if (!t) return fail(NE_ERR_NOMEM, "host allocation failed");
    if (init) {
        hipStream_t st = static_cast<hipStream_t>(hip_stream);
        const int64_t total = num_nodes * (dim / 4);
        const int64_t want = (total + 255) / 256;
        const unsigned grid = static_cast<unsigned>(want < 65536 * 4 ? (want > 0 ? want : 1) : 65536 * 4);
        hipLaunchKernelGGL(init_tables_kernel, dim3(grid), dim3(256), 0, st, reinterpret_cast<float4*>(vertex_dev),
                           reinterpret_cast<float4*>(context_dev), num_nodes, dim / 4, static_cast<float>(dim),
                           static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32));
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) {
            delete t;
            return fail(NE_ERR_HIP, std::string("init_tables launch: ") + hipGetErrorString(e));
        }
    }
    *out = t;
    return NE_OK;
}

void ne_destroy_tables(ne_tables* t) { delete t; }
void ne_destroy_alias(ne_alias* a) { delete a; }

ne_status ne_build_neg_alias(ne_alias** out, const uint32_t* degree_host, int64_t n, int32_t base,
                             void* alias_dev, void* hip_stream)
{
    if (!out) return fail(NE_ERR_ARG, "out is NULL");
    *out = nullptr;
    if (!degree_host || !alias_dev) return fail(NE_ERR_ARG, "degree_host or alias_dev is NULL");
    if (n <= 0 || base < 0 || static_cast<int64_t>(base) + n >= (static_cast<int64_t>(1) << 31))
        return fail(NE_ERR_ARG, "need 0 < n, 0 <= base, base + n < 2^31");
    if (!aligned(alias_dev, 8)) return fail(NE_ERR_ARG, "alias_dev must be 8-byte aligned");

    // weights deg^0.75 and their plain left-to-right sum
    std::vector<double> prob;
    std::vector<int64_t> lo_stack, hi_stack;
    uint2* staged = nullptr;
    try {
        prob.resize(static_cast<size_t>(n));
        lo_stack.reserve(static_cast<size_t>(n));
        hi_stack.reserve(static_cast<size_t>(n));
    } catch (const std::bad_alloc&) {
        return fail(NE_ERR_NOMEM, "host allocation failed");
    }
    double total = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        const double dg = static_cast<double>(degree_host[i]);
        const double w = std::sqrt(dg) * std::sqrt(std::sqrt(dg));
        prob[i] = w;
        total += w;
    }
    if (!(total > 0.0)) return fail(NE_ERR_ARG, "all degrees are zero");
    const double nn = static_cast<double>(n);
    for (int64_t i = 0; i < n; ++i) {
        prob[i] = (prob[i] * nn) / total;
        (prob[i] < 1.0 ? lo_stack : hi_stack).push_back(i);
    }
    NE_HIP_CHECK(hipHostMalloc(reinterpret_cast<void**>(&staged), static_cast<size_t>(n) * sizeof(uint2), hipHostMallocDefault));
    auto quantise = [](double thr) -> uint32_t {
        double q = std::floor(thr * 4294967296.0);
        if (q > 4294967295.0) q = 4294967295.0;
        if (q < 0.0) q = 0.0;
        return static_cast<uint32_t>(q);
    };
    // Vose: pair the most recently pushed under-full entry with the most recently pushed over-full one
    while (!lo_stack.empty() && !hi_stack.empty()) {
        const int64_t s = lo_stack.back(); lo_stack.pop_back();
        const int64_t l = hi_stack.back(); hi_stack.pop_back();
        staged[s] = make_uint2(quantise(prob[s]), static_cast<uint32_t>(l));
        prob[l] = (prob[l] + prob[s]) - 1.0;
        (prob[l] < 1.0 ? lo_stack : hi_stack).push_back(l);
    }
    for (int64_t l : hi_stack) staged[l] = make_uint2(0xFFFFFFFFu, static_cast<uint32_t>(l));
    for (int64_t s : lo_stack) staged[s] = make_uint2(0xFFFFFFFFu, static_cast<uint32_t>(s));

    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    hipError_t e = hipMemcpyAsync(alias_dev, staged, static_cast<size_t>(n) * sizeof(uint2), hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    (void)hipHostFree(staged);
    if (e != hipSuccess) return fail(NE_ERR_HIP, std::string("alias copy: ") + hipGetErrorString(e));

    ne_alias* a = new (std::nothrow) ne_alias{static_cast<const uint2*>(alias_dev), n, base};
    if (!a) return fail(NE_ERR_NOMEM, "host allocation failed");
    *out = a;
    return NE_OK;
}

size_t ne_staging_bytes(int64_t B, int32_t dim, int32_t K)
{
    if (B < 0 || B > kMaxBatch || dim < 4 || dim > NE_MAX_DIM || dim % 4 != 0 || K < 0 || K > NE_MAX_NEGATIVES)
        return 0;
    return staging_layout(B > 0 ? B : 1, dim, K).total;
}

ne_status ne_train_batch(ne_tables* t, const ne_alias* al, const int32_t* pairs_dev, int64_t B, int32_t K,
                         float lr, uint64_t sample_base, void* staging_dev, size_t staging_bytes,
                         int32_t* neg_out_dev, void* hip_stream)
{
    Shape shape;
    ne_status rc = check_batch_args(t, al, pairs_dev, B, K, &shape);
    if (rc != NE_OK) return rc;
    if (!std::isfinite(lr)) return fail(NE_ERR_ARG, "lr is not finite");
    if (B == 0) return NE_OK;
    const StagingLayout L = staging_layout(B, t->dim, K);
    if (!staging_dev || !aligned(staging_dev, 16)) return fail(NE_ERR_ARG, "staging_dev is NULL or not 16-byte aligned");
    if (staging_bytes < L.total) return fail(NE_ERR_ARG, "staging buffer smaller than ne_staging_bytes(B, dim, K)");

    char* sp = static_cast<char*>(staging_dev);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    ScoreArgs sa{};
    sa.X = reinterpret_cast<const float4*>(t->vertex);
    sa.C = reinterpret_cast<const float4*>(t->context);
    sa.pairs = reinterpret_cast<const int2*>(pairs_dev);
    sa.B = B; sa.K = K; sa.d4 = t->dim / 4; sa.lr = lr; sa.sample_base = sample_base;
    sa.k0 = static_cast<uint32_t>(t->seed); sa.k1 = static_cast<uint32_t>(t->seed >> 32);
    sa.alias = al ? al->table : nullptr; sa.alias_n = al ? static_cast<uint64_t>(al->n) : 1; sa.alias_base = al ? al->base : 0;
    sa.gbuf = reinterpret_cast<float*>(sp + L.g_off);
    sa.nbuf = reinterpret_cast<int32_t*>(sp + L.n_off);
    sa.xbuf = reinterpret_cast<float4*>(sp + L.x_off);
    sa.dxbuf = reinterpret_cast<float4*>(sp + L.dx_off);
    sa.neg_out = neg_out_dev; sa.loss = nullptr;
    hipError_t e = launch_score<true>(shape, sa, st);
    if (e != hipSuccess) return fail(NE_ERR_HIP, std::string("score launch: ") + hipGetErrorString(e));

    UpdateArgs ua{};
    ua.X = t->vertex; ua.C = t->context; ua.pairs = sa.pairs; ua.B = B; ua.K = K; ua.d4 = sa.d4;
    ua.gbuf = sa.gbuf; ua.nbuf = sa.nbuf; ua.xbuf = sa.xbuf; ua.dxbuf = sa.dxbuf;
    e = launch_update(shape, ua, st);
    if (e != hipSuccess) return fail(NE_ERR_HIP, std::string("update launch: ") + hipGetErrorString(e));
    return NE_OK;
}

ne_status ne_eval_loss(const ne_tables* t, const ne_alias* al, const int32_t* pairs_dev, int64_t B, int32_t K,
                       uint64_t sample_base, double* loss_sum_dev, int32_t* neg_out_dev, void* hip_stream)
{
    Shape shape;
    ne_status rc = check_batch_args(t, al, pairs_dev, B, K, &shape);
    if (rc != NE_OK) return rc;
    if (!loss_sum_dev || !aligned(loss_sum_dev, 8)) return fail(NE_ERR_ARG, "loss_sum_dev is NULL or misaligned");
    if (B == 0) return NE_OK;
    ScoreArgs sa{};
    sa.X = reinterpret_cast<const float4*>(t->vertex);
    sa.C = reinterpret_cast<const float4*>(t->context);
    sa.pairs = reinterpret_cast<const int2*>(pairs_dev);
    sa.B = B; sa.K = K; sa.d4 = t->dim / 4; sa.lr = 0.0f; sa.sample_base = sample_base;
    sa.k0 = static_cast<uint32_t>(t->seed); sa.k1 = static_cast<uint32_t>(t->seed >> 32);
    sa.alias = al ? al->table : nullptr; sa.alias_n = al ? static_cast<uint64_t>(al->n) : 1; sa.alias_base = al ? al->base : 0;
    sa.neg_out = neg_out_dev; sa.loss = loss_sum_dev;
    hipError_t e = launch_score<false>(shape, sa, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail(NE_ERR_HIP, std::string("eval launch: ") + hipGetErrorString(e));
    return NE_OK;
}

ne_status ne_validate_pairs(const ne_tables* t, const int32_t* pairs_dev, int64_t B,
                            unsigned long long* bad_count_dev, void* hip_stream)
{
    if (!t || !bad_count_dev) return fail(NE_ERR_ARG, "NULL argument");
    if (B < 0 || B > kMaxBatch * 16) return fail(NE_ERR_ARG, "B out of range");
    if (B == 0) return NE_OK;
    if (!pairs_dev) return fail(NE_ERR_ARG, "pairs_dev is NULL");
    const int64_t count = 2 * B;
    const int64_t want = (count + 255) / 256;
    const unsigned grid = static_cast<unsigned>(want < 65536 ? want : 65536);
    hipLaunchKernelGGL(validate_pairs_kernel, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(hip_stream), pairs_dev,
                       count, t->num_nodes, bad_count_dev);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(NE_ERR_HIP, std::string("validate launch: ") + hipGetErrorString(e));
    return NE_OK;
}

}  // extern "C"
