// SGNS node-embedding training for MI355X (gfx950): HIP kernels and the C ABI declared in ne.h.
//
// One batch of the embedding-training loop (Algorithm 1; Sec. II-A "Training Process") has four
// phases:
//
//   claim, resolve (ids only)  one thread per row reference (src, ctx and the K negatives of every
//          pair).  claim draws the negative (Philox + alias table) and stores (key, reference
//          index) at the key's hash position with a plain 8-byte store; whichever store lands last
//          owns the position.  resolve reads the position back: a reference whose key owns it but
//          whose index differs has found a second reference of the same row and flags the row as
//          shared; references whose key lost the position (a different row hashed there) fall back
//          to compare-and-swap probing.  Returning atomics retire slowly on this chip, so only that
//          minority uses them.
//   train  one lane group per pair: gathers x = vertex[src] and the K+1 context rows (dwordx4),
//          reduces the K+1 dot products with DPP, forms g_j and the deltas.  A row that only this
//          pair names is rewritten in place from registers (old + delta, one plain store: the row
//          costs one read and one write).  A shared row is left untouched - other pairs must still
//          read its pre-batch value - and its delta is added to the row's slot (indexed by hash
//          position) with fp32 atomics.  Where most rows are shared the atomics' rate would bound
//          the kernel; there the first references to arrive at a row (ranked by a returning
//          counter, which is cheap) instead store their delta with plain stores in a buffer row
//          of their own and enter the row's member list.
//   apply  adds each shared row's slot, and the buffer rows of its member list, to the table row,
//          zeroes the slot and the counter; the hash positions of the batch are emptied.
//
// This is exactly minibatch-synchronous: no row that a second reference could read is written
// before the apply phase, and all contributions to a row are summed.  fp32 atomics on gfx950
// retire one dword per L2 channel clock, far below the rate of plain row stores, which is why only
// shared rows go through them.
//
// claim and resolve never touch the tables, so for a run of batches (ne_train_block) they ride
// along in the kernels of the batch before: kernel A = train(t) + claim(t+1), kernel B = apply(t) +
// resolve(t+1), two launches per batch, with two sets of hash state used alternately.
//
// The same four phases serve three shapes of batch: pairs (ne_train_batch, ne_train_block), and walks
// (ne_train_walks: on-device augmentation) by entries or by segments, which differ only in how the
// references are laid out (claim) and in what a lane group or workgroup keeps on chip (train).
// Beside the exact step: the per-sample mode (ne_train_block_async: the same launches, but a shared
// row's deltas are added to the table row itself with atomics while other pairs may still read it, and
// the apply phase has no row work), the loss and pair-score kernels for evaluation, and table
// initialisation.
#include "ne_internal.h"

static thread_local std::string g_last_error;

ne_status fail(ne_status st, const std::string& msg)
{
    g_last_error = msg;
    return st;
}

namespace {

// ---------------------------------------------------------------------------------------------
// small fills (hipMemsetAsync is avoided so that callers may capture the stream)
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void fill_u32_kernel(uint32_t* __restrict__ p, size_t n, uint32_t v)
{
    const size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
    for (size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = v;
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
// claim + resolve kernels: one thread per row reference.  Reference j of pair b: j = 0 the source
// row (vertex table), j = 1 the positive context row, j = 2.. negative j-2 (context table).
// key = row | (context table ? 1 << 31 : 0).
// ---------------------------------------------------------------------------------------------
constexpr unsigned long long kEmptySlot = ~0ull;

__device__ __forceinline__ uint32_t hash_key(uint32_t key, uint32_t mask) { return hash_position(key, mask); }

struct PrepArgs {
    const int2* pairs;    // pair mode: the batch's pairs
    const int32_t* walks; // walk mode (pairs == nullptr): the batch's walks, int32 [..][walk_len]
    int32_t walk_len, window;
    uint32_t refs;        // references of the batch; 0 = nothing to prepare
    uint32_t R;           // references per pair (K + 2) / per walk entry (1 + window * (K + 1)) / per walk segment
    uint32_t xrefs;       // how many references at the front of each group of R name the vertex table (1; segment mode: entries per segment)
    uint32_t seg_entries; // walk mode: 0 = one reference group per walk entry; else entries per segment
    uint32_t segs_per_walk;
    int32_t K;
    uint64_t sample_base;
    uint32_t k0, k1;
    const uint2* alias;
    uint64_t alias_n;
    int32_t alias_base;
    unsigned long long* slots;
    uint32_t mask;        // cap - 1
    uint8_t* shared;      // per hash position: the row there is named more than once (what the apply sweep reads)
    uint8_t* refshared;   // per reference: the same fact, where the train kernel reads it without a dependent lookup
    int32_t* ids;
    uint32_t* posbuf;
    int32_t* neg_out;
    // sample prefetch riding along (ne_train_block_pinned): fetch_blocks helper workgroups copy fetch_n
    // pairs from pinned host memory (fetch_src: its device address) into the staging ring (fetch_dst)
    const int2* fetch_src;
    int2* fetch_dst;
    int64_t fetch_n;
    uint32_t fetch_blocks;
};

// Both phases are chains of dependent memory accesses with next to no arithmetic, so each thread
// runs kPrepUnroll references at once: a block covers 256 * kPrepUnroll consecutive references.
constexpr int kPrepUnroll = 4;

__device__ __forceinline__ void claim_pair_refs(const PrepArgs& a, unsigned block, unsigned tid)
{
    const uint32_t R = a.R;
    uint32_t t[kPrepUnroll], b[kPrepUnroll];
    int j[kPrepUnroll];
    int32_t id[kPrepUnroll];
    uint4 rnd[kPrepUnroll];
    uint2 entry[kPrepUnroll];
    uint64_t draw_slot[kPrepUnroll];
#pragma unroll
    for (int u = 0; u < kPrepUnroll; ++u) {
        t[u] = (block * kPrepUnroll + u) * 256u + tid;
        b[u] = t[u] / R;
        j[u] = static_cast<int>(t[u] - b[u] * R);
        id[u] = 0;
        if (t[u] < a.refs) {
            if (j[u] < 2) {
                const int2 pr = a.pairs[b[u]];
                id[u] = j[u] == 0 ? pr.x : pr.y;
            } else {
                const uint64_t sample = a.sample_base + b[u];
                rnd[u] = philox4x32_10(make_uint4(static_cast<uint32_t>(sample), static_cast<uint32_t>(sample >> 32),
                                                  static_cast<uint32_t>(j[u] - 2), kStreamNegative), a.k0, a.k1);
                draw_slot[u] = __umul64hi((static_cast<uint64_t>(rnd[u].x) << 32) | rnd[u].y, a.alias_n);
                entry[u] = a.alias[draw_slot[u]];
            }
        }
    }
#pragma unroll
    for (int u = 0; u < kPrepUnroll; ++u) {
        if (t[u] < a.refs) {
            if (j[u] >= 2) {
                id[u] = a.alias_base + static_cast<int32_t>(rnd[u].z < entry[u].x ? static_cast<uint32_t>(draw_slot[u]) : entry[u].y);
                if (a.neg_out) a.neg_out[static_cast<int64_t>(b[u]) * a.K + (j[u] - 2)] = id[u];
            }
            a.ids[t[u]] = id[u];
            a.refshared[t[u]] = 0;   // resolve sets it, one launch later
            const uint32_t key = static_cast<uint32_t>(id[u]) | (j[u] == 0 ? 0u : 0x80000000u);
            a.slots[hash_key(key, a.mask)] = (static_cast<unsigned long long>(key) << 32) | t[u];
        }
    }
}

// Walk mode (on-device augmentation, Algorithm 1 "network augmentation"): the batch is a set of
// walks int32 [n][L]; position i of a walk is the source of the pairs (walk[i], walk[i+j]),
// 1 <= j <= window, that exist (both entries non-negative, i + j < L).  References of position p:
//   0                          the source row (vertex table), present if the position has a pair
//   1 + (j-1)(K+1)             the context row of pair j
//   1 + (j-1)(K+1) + 1 + k     negative k of pair j, drawn for sample index sample_base + p*window + (j-1)
// Absent references get id -1 and claim nothing.
__device__ __forceinline__ void claim_walk_refs(const PrepArgs& a, unsigned block, unsigned tid)
{
    const uint32_t R = a.R;
    const uint32_t L = static_cast<uint32_t>(a.walk_len), W = static_cast<uint32_t>(a.window), K1 = static_cast<uint32_t>(a.K + 1);
    uint32_t t[kPrepUnroll], p[kPrepUnroll], jj[kPrepUnroll];
    int kk[kPrepUnroll];     // -2: source, -1: context, >= 0: negative k
    int32_t id[kPrepUnroll];
    bool valid[kPrepUnroll];
    uint4 rnd[kPrepUnroll];
    uint2 entry[kPrepUnroll];
    uint64_t draw_slot[kPrepUnroll];
#pragma unroll
    for (int u = 0; u < kPrepUnroll; ++u) {
        t[u] = (block * kPrepUnroll + u) * 256u + tid;
        id[u] = -1;
        valid[u] = false;
        kk[u] = -2;
        jj[u] = 0;
        p[u] = 0;
        if (t[u] < a.refs) {
            p[u] = t[u] / R;
            const uint32_t q = t[u] - p[u] * R;
            const uint32_t r = p[u] / L, i = p[u] - r * L;
            const int32_t* wk = a.walks + static_cast<int64_t>(r) * L;
            const int32_t src = wk[i];
            if (q == 0) {
                bool has = false;
                for (uint32_t j = 1; j <= W && i + j < L; ++j) has = has || wk[i + j] >= 0;
                valid[u] = src >= 0 && has;
                id[u] = src;
            } else {
                jj[u] = (q - 1) / K1;
                kk[u] = static_cast<int>(q - 1 - jj[u] * K1) - 1;
                const uint32_t c = i + jj[u] + 1;
                const int32_t ctx = c < L ? wk[c] : -1;
                valid[u] = src >= 0 && ctx >= 0;
                id[u] = ctx;
                if (valid[u] && kk[u] >= 0) {
                    const uint64_t sample = a.sample_base + static_cast<uint64_t>(p[u]) * W + jj[u];
                    rnd[u] = philox4x32_10(make_uint4(static_cast<uint32_t>(sample), static_cast<uint32_t>(sample >> 32),
                                                      static_cast<uint32_t>(kk[u]), kStreamNegative), a.k0, a.k1);
                    draw_slot[u] = __umul64hi((static_cast<uint64_t>(rnd[u].x) << 32) | rnd[u].y, a.alias_n);
                    entry[u] = a.alias[draw_slot[u]];
                }
            }
        }
    }
#pragma unroll
    for (int u = 0; u < kPrepUnroll; ++u) {
        if (t[u] >= a.refs) continue;
        if (valid[u] && kk[u] >= 0) {
            id[u] = a.alias_base + static_cast<int32_t>(rnd[u].z < entry[u].x ? static_cast<uint32_t>(draw_slot[u]) : entry[u].y);
            if (a.neg_out) a.neg_out[(static_cast<int64_t>(p[u]) * W + jj[u]) * a.K + kk[u]] = id[u];
        }
        if (!valid[u]) id[u] = -1;
        a.ids[t[u]] = id[u];
        a.refshared[t[u]] = 0;
        if (valid[u]) {
            const uint32_t key = static_cast<uint32_t>(id[u]) | (kk[u] == -2 ? 0u : 0x80000000u);
            a.slots[hash_key(key, a.mask)] = (static_cast<unsigned long long>(key) << 32) | t[u];
        }
    }
}

// Walk mode by segments: a walk is cut into segments of E = seg_entries consecutive entries, one
// workgroup of the train kernel each.  The workgroup sums on chip everything its entries contribute
// to each other, so a segment names every row once.  References of segment (walk r, entries p0 ..
// p0+E-1), CT = E + window - 1:
//   q < E                    vertex row of entry p0 + q, present if that entry starts a sample
//   E <= q < E + CT          context row of entry p0 + 1 + (q - E), present if one of the segment's
//                            entries has it as a sample's context (the last window-1 of them belong
//                            to the next segment's entries too: both segments name them)
//   E + CT + (e*window + j-1)*K + k   negative k of sample (entry p0 + e, offset j)
__device__ __forceinline__ void claim_seg_refs(const PrepArgs& a, unsigned block, unsigned tid)
{
    const uint32_t R = a.R, E = a.seg_entries;
    const uint32_t L = static_cast<uint32_t>(a.walk_len), W = static_cast<uint32_t>(a.window), K = static_cast<uint32_t>(a.K);
    const uint32_t CT = E + W - 1;
    uint32_t t[kPrepUnroll], samp[kPrepUnroll];
    int kk[kPrepUnroll];     // -2: vertex row, -1: context row, >= 0: negative k
    int32_t id[kPrepUnroll];
    bool valid[kPrepUnroll];
    uint4 rnd[kPrepUnroll];
    uint2 entry[kPrepUnroll];
    uint64_t draw_slot[kPrepUnroll];
#pragma unroll
    for (int u = 0; u < kPrepUnroll; ++u) {
        t[u] = (block * kPrepUnroll + u) * 256u + tid;
        id[u] = -1;
        valid[u] = false;
        kk[u] = -2;
        samp[u] = 0;
        if (t[u] < a.refs) {
            const uint32_t seg = t[u] / R, q = t[u] - seg * R;
            const uint32_t r = seg / a.segs_per_walk, p0 = (seg - r * a.segs_per_walk) * E;
            const int32_t* wk = a.walks + static_cast<int64_t>(r) * L;
            if (q < E) {
                const uint32_t i = p0 + q;
                if (i < L) {
                    bool has = false;
                    for (uint32_t j = 1; j <= W && i + j < L; ++j) has = has || wk[i + j] >= 0;
                    id[u] = wk[i];
                    valid[u] = id[u] >= 0 && has;
                }
            } else if (q < E + CT) {
                kk[u] = -1;
                const uint32_t c = p0 + 1 + (q - E);
                if (c < L) {
                    // sources of this segment that have entry c inside their window
                    const uint32_t lo = c > p0 + W ? c - W : p0, hi = (c - 1 < p0 + E - 1) ? c - 1 : p0 + E - 1;
                    bool has = false;
                    for (uint32_t i = lo; i <= hi; ++i) has = has || wk[i] >= 0;
                    id[u] = wk[c];
                    valid[u] = id[u] >= 0 && has;
                }
            } else {
                const uint32_t n = q - E - CT, pj = n / K;    // pj = e * W + (j - 1)
                kk[u] = static_cast<int>(n - pj * K);
                const uint32_t e = pj / W, j = pj - e * W + 1, i = p0 + e;
                if (i + j < L) {
                    valid[u] = wk[i] >= 0 && wk[i + j] >= 0;
                    samp[u] = (r * L + i) * W + (j - 1);
                    if (valid[u]) {
                        const uint64_t sample = a.sample_base + samp[u];
                        rnd[u] = philox4x32_10(make_uint4(static_cast<uint32_t>(sample), static_cast<uint32_t>(sample >> 32),
                                                          static_cast<uint32_t>(kk[u]), kStreamNegative), a.k0, a.k1);
                        draw_slot[u] = __umul64hi((static_cast<uint64_t>(rnd[u].x) << 32) | rnd[u].y, a.alias_n);
                        entry[u] = a.alias[draw_slot[u]];
                    }
                }
            }
        }
    }
#pragma unroll
    for (int u = 0; u < kPrepUnroll; ++u) {
        if (t[u] >= a.refs) continue;
        if (valid[u] && kk[u] >= 0) {
            id[u] = a.alias_base + static_cast<int32_t>(rnd[u].z < entry[u].x ? static_cast<uint32_t>(draw_slot[u]) : entry[u].y);
            if (a.neg_out) a.neg_out[static_cast<int64_t>(samp[u]) * a.K + kk[u]] = id[u];
        }
        if (!valid[u]) id[u] = -1;
        a.ids[t[u]] = id[u];
        a.refshared[t[u]] = 0;
        if (valid[u]) {
            const uint32_t key = static_cast<uint32_t>(id[u]) | (kk[u] == -2 ? 0u : 0x80000000u);
            a.slots[hash_key(key, a.mask)] = (static_cast<unsigned long long>(key) << 32) | t[u];
        }
    }
}

__device__ __forceinline__ void claim_refs(const PrepArgs& a, unsigned block, unsigned tid)
{
    if (a.pairs) claim_pair_refs(a, block, tid);
    else if (a.seg_entries) claim_seg_refs(a, block, tid);
    else claim_walk_refs(a, block, tid);
}

__device__ __forceinline__ void resolve_refs(const PrepArgs& a, unsigned block)
{
    const uint32_t R = a.R;
    uint32_t t[kPrepUnroll], key[kPrepUnroll], pos[kPrepUnroll];
    bool live[kPrepUnroll];   // walk mode leaves holes (id -1) where a walk has no pair
    unsigned long long owner[kPrepUnroll];
#pragma unroll
    for (int u = 0; u < kPrepUnroll; ++u) {
        t[u] = (block * kPrepUnroll + u) * 256u + threadIdx.x;
        key[u] = 0;
        live[u] = false;
        if (t[u] < a.refs) {
            const int32_t id = a.ids[t[u]];
            live[u] = id >= 0;
            key[u] = static_cast<uint32_t>(id) | ((t[u] % R) < a.xrefs ? 0u : 0x80000000u);
        }
    }
#pragma unroll
    for (int u = 0; u < kPrepUnroll; ++u) {
        pos[u] = hash_key(key[u], a.mask);
        owner[u] = live[u] ? a.slots[pos[u]] : 0ull;
    }
#pragma unroll
    for (int u = 0; u < kPrepUnroll; ++u) {
        if (!live[u]) continue;
        uint32_t p = pos[u];
        if (static_cast<uint32_t>(owner[u] >> 32) == key[u]) {
            // my row owns its home position; any reference but the one whose store landed last
            // proves that the row is named at least twice
            if (static_cast<uint32_t>(owner[u]) != t[u]) {
                a.shared[p] = 1;
                a.refshared[t[u]] = 1;
                a.refshared[static_cast<uint32_t>(owner[u])] = 1;   // the owner cannot tell by itself
            }
        } else {
            // another row owns the home position: probe onwards.  Positions only ever go from empty
            // to occupied here, and the table holds at most half as many keys as positions, so the walk ends.
            const unsigned long long mine = (static_cast<unsigned long long>(key[u]) << 32) | t[u];
            while (true) {
                p = (p + 1) & a.mask;
                const unsigned long long prev = atomicCAS(&a.slots[p], kEmptySlot, mine);
                if (prev == kEmptySlot) break;
                if (static_cast<uint32_t>(prev >> 32) == key[u]) {
                    a.shared[p] = 1;
                    a.refshared[t[u]] = 1;
                    a.refshared[static_cast<uint32_t>(prev)] = 1;
                    break;
                }
            }
        }
        a.posbuf[t[u]] = p;
    }
}

// Number of blocks either phase needs for `refs` references.
inline unsigned prep_blocks(uint32_t refs) { return (refs + 256u * kPrepUnroll - 1u) / (256u * kPrepUnroll); }

// ---------------------------------------------------------------------------------------------
// sample prefetch (ne_train_block_pinned): a few workgroups copy the pairs of a later batch from
// pinned host memory, which they read directly, into a device staging ring.  They ride inside the
// training launches; the first two batches of a call use the stand-alone kernel.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void fetch_pairs(const int2* __restrict__ src, int2* __restrict__ dst, int64_t n, int64_t i0,
                                            int64_t stride)
{
    // pairs two at a time while both buffers allow 16-byte accesses
    const bool wide = ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15) == 0;
    if (wide) {
        const int64_t n2 = n / 2;
        const int4* s4 = reinterpret_cast<const int4*>(src);
        int4* d4 = reinterpret_cast<int4*>(dst);
        // four loads in flight per thread: the link's latency is long and the copy should stay small
        int64_t i = i0;
        for (; i + 3 * stride < n2; i += 4 * stride) {
            const int4 v0 = s4[i], v1 = s4[i + stride], v2 = s4[i + 2 * stride], v3 = s4[i + 3 * stride];
            d4[i] = v0; d4[i + stride] = v1; d4[i + 2 * stride] = v2; d4[i + 3 * stride] = v3;
        }
        for (; i < n2; i += stride) d4[i] = s4[i];
        if (i0 == 0 && (n & 1)) dst[n - 1] = src[n - 1];
    } else {
        for (int64_t i = i0; i < n; i += stride) dst[i] = src[i];
    }
}

__global__ __launch_bounds__(256) void fetch_pairs_kernel(const int2* __restrict__ src, int2* __restrict__ dst, int64_t n)
{
    fetch_pairs(src, dst, n, static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x,
                static_cast<int64_t>(gridDim.x) * blockDim.x);
}

// Placement of `extra` helper blocks among `total` blocks of a fused launch: every period-th block is
// a helper until they run out, so helpers and main blocks are resident together from the start.
__device__ __forceinline__ bool fused_block(unsigned extra, unsigned period, unsigned* index)
{
    const unsigned i = blockIdx.x;
    if (extra && i % period == 0 && i / period < extra) { *index = i / period; return true; }
    const unsigned before = extra ? min(extra, (i + period - 1) / period) : 0u;
    *index = i - before;
    return false;
}

__global__ __launch_bounds__(256) void claim_kernel(PrepArgs a) { claim_refs(a, blockIdx.x, threadIdx.x); }
__global__ __launch_bounds__(256) void resolve_kernel(PrepArgs a) { resolve_refs(a, blockIdx.x); }

// ---------------------------------------------------------------------------------------------
// train kernel.  G lanes per pair, NCH float4 chunks per lane (chunk index = lg + i*G, valid while
// < d4), JB context rows in flight at a time.
// ---------------------------------------------------------------------------------------------
struct TrainArgs {
    float4* X;
    float4* C;
    int64_t B;            // pairs (pair mode) / walk positions (walk mode)
    int32_t window;       // walk mode: pairs per position
    int32_t K;
    int32_t d4;
    float lr;
    const int32_t* ids;
    const uint32_t* posbuf;
    const uint8_t* refshared;   // per reference: its row is named by another reference too
    float* delta;
    // shared rows, list path: the first list_cap references to arrive at a row (0 = path off)
    uint32_t list_cap;
    uint32_t* count;      // [positions] references of the row that have arrived (zero between batches)
    uint32_t* members;    // [positions][kListCap] reference indices of the first arrivals
    float4* dbuf;         // [references][d4] their deltas
    // per-sample mode (ne_train_block_async): a shared row's deltas go straight to the table row with atomics
    // instead of to a slot, so pairs that read the row later see them; nothing is left for the apply phase
    int32_t direct;
};

// Longest member list of a shared row.
constexpr uint32_t kListCap = 8;

// Rank of a reference among those arriving at its shared row (~0 with the list path off).  The
// returning atomic is cheap next to a row's traffic and is issued early, so its latency hides
// behind the row gathers.
template <int G>
__device__ __forceinline__ uint32_t arrival_rank(const TrainArgs& a, uint32_t pos, int lg)
{
    uint32_t r = ~0u;
    if (a.list_cap) {
        if (lg == 0) r = atomicAdd(&a.count[pos], 1u);
        r = __shfl(r, 0, G);
    }
    return r;
}

// Element e = lg + m*G of a row, for m < 4*NCH: the layout in which one atomic instruction of a lane
// group covers consecutive dwords.  The float4-chunk layout is turned into it through LDS.
template <int G, int NCH>
__device__ __forceinline__ void to_consecutive(const float4 (&v)[NCH], float (&out)[4 * NCH], float* lds_row, int lg)
{
#pragma unroll
    for (int i = 0; i < NCH; ++i) reinterpret_cast<float4*>(lds_row)[lg + i * G] = v[i];
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int m = 0; m < 4 * NCH; ++m) out[m] = lds_row[lg + m * G];
    __builtin_amdgcn_wave_barrier();
}

// Delta dv of reference `ref` to the shared row at hash position pos.  A reference that arrived among
// the first list_cap stores it with plain stores in its own row of dbuf and enters the row's member
// list (the apply kernel sums the list); a later one adds it to the row's slot with atomics, which
// retire one dword per memory channel clock and would otherwise bound batches with many shared rows.
template <int G, int NCH>
__device__ __forceinline__ void shared_row_delta(const TrainArgs& a, uint32_t pos, uint32_t ref, uint32_t rank,
                                                 const float4 (&dv)[NCH], float* lds_row, int lg, int d4, float4* row)
{
    if (rank < a.list_cap) {
        float4* out = a.dbuf + static_cast<int64_t>(ref) * d4;
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int ci = lg + i * G;
            if (ci < d4) out[ci] = dv[i];
        }
        if (lg == 0) a.members[static_cast<int64_t>(pos) * kListCap + rank] = ref;
    } else {
        float t[4 * NCH];
        to_consecutive<G, NCH>(dv, t, lds_row, lg);
        float* slot = a.direct ? reinterpret_cast<float*>(row) : a.delta + static_cast<int64_t>(pos) * (d4 * 4);
#pragma unroll
        for (int m = 0; m < 4 * NCH; ++m) {
            const int e = lg + m * G;
            if (e < d4 * 4) unsafeAtomicAdd(slot + e, t[m]);
        }
    }
}

// K+1 context rows of one pair (rows 0..K; with POS_FIRST row 0 is the positive, every other row a
// negative), JB at a time: gather, score against x, form g_j, add g_j c_j to dx, and update the row:
// rewritten in place if only this reference names it, else its delta goes to the reference's buffer
// row (list path, first arrivals) or to the row's slot with atomics.  Lane j + LANE0 of the group holds
// reference j's id, hash position, shared flag and index in the batch.
template <int G, int NCH, int JB, int LANE0, bool POS_FIRST = true>
__device__ __forceinline__ void context_rows_of_pair(const TrainArgs& a, int K, int d4, int d, const float4 (&xr)[NCH],
                                                     const float (&xt)[4 * NCH], float4 (&dx)[NCH], int32_t id_mine,
                                                     uint32_t pos_mine, int shared_mine, uint32_t ref_mine, int lg)
{
    // ranks of this pair's references to shared rows, all in one returning atomic
    uint32_t rank_mine = ~0u;
    if (a.list_cap && shared_mine) rank_mine = atomicAdd(&a.count[pos_mine], 1u);
    for (int j0 = 0; j0 <= K; j0 += JB) {
        float4 cr[JB][NCH];
        float part[JB];
        float4* crow[JB];
#pragma unroll
        for (int jj = 0; jj < JB; ++jj) {
            const int j = j0 + jj;
            const int32_t id = __shfl(id_mine, (j <= K ? j : K) + LANE0, G);
            crow[jj] = a.C + static_cast<int64_t>(id) * d4;
#pragma unroll
            for (int i = 0; i < NCH; ++i) {
                const int ci = lg + i * G;
                cr[jj][i] = (j <= K && ci < d4) ? crow[jj][ci] : make_float4(0.f, 0.f, 0.f, 0.f);
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
                const float sg = sigmoidf(part[jj]);
                const float g = a.lr * ((POS_FIRST && j == 0) ? 1.0f - sg : -sg);
                const int shared = __shfl(shared_mine, j + LANE0, G);
                const uint32_t pos = __shfl(pos_mine, j + LANE0, G);
                const uint32_t rank = __shfl(rank_mine, j + LANE0, G);
                const uint32_t ref = __shfl(ref_mine, j + LANE0, G);
#pragma unroll
                for (int i = 0; i < NCH; ++i) dx[i] = axpy4(g, cr[jj][i], dx[i]);
                if (!shared) {
#pragma unroll
                    for (int i = 0; i < NCH; ++i) {
                        const int ci = lg + i * G;
                        if (ci < d4) crow[jj][ci] = axpy4(g, xr[i], cr[jj][i]);
                    }
                } else if (rank < a.list_cap) {
                    float4* out = a.dbuf + static_cast<int64_t>(ref) * d4;
#pragma unroll
                    for (int i = 0; i < NCH; ++i) {
                        const int ci = lg + i * G;
                        if (ci < d4) out[ci] = make_float4(g * xr[i].x, g * xr[i].y, g * xr[i].z, g * xr[i].w);
                    }
                    if (lg == 0) a.members[static_cast<int64_t>(pos) * kListCap + rank] = ref;
                } else {
                    float* slot = a.direct ? reinterpret_cast<float*>(crow[jj]) : a.delta + static_cast<int64_t>(pos) * d;
#pragma unroll
                    for (int m = 0; m < 4 * NCH; ++m) {
                        const int e = lg + m * G;
                        if (e < d) unsafeAtomicAdd(slot + e, g * xt[m]);
                    }
                }
            }
        }
    }

}

#ifndef NE_TRAIN_THREADS
#define NE_TRAIN_THREADS 256
#endif
constexpr int kTrainThreads = NE_TRAIN_THREADS;   // threads per block of the train kernel (a claim block's 256-thread share is looped)

template <int G, int NCH, int JB>
__global__ __launch_bounds__(kTrainThreads) void train_kernel(TrainArgs a, PrepArgs next, unsigned claim_blocks, unsigned period)
{
    constexpr int GROUPS = kTrainThreads / G;
    __shared__ float lds[GROUPS][4 * G * NCH];
    // some blocks do the id-only claim phase of the next batch
    unsigned block;
    if (fused_block(claim_blocks, period, &block)) {
        if (block < next.fetch_blocks) {   // sample prefetch for the batch after the next
            fetch_pairs(next.fetch_src, next.fetch_dst, next.fetch_n, static_cast<int64_t>(block) * kTrainThreads + threadIdx.x,
                        static_cast<int64_t>(next.fetch_blocks) * kTrainThreads);
            return;
        }
        block -= next.fetch_blocks;
        for (unsigned tid = threadIdx.x; tid < 256u; tid += kTrainThreads) claim_refs(next, block, tid);
        return;
    }
    const int lg = threadIdx.x & (G - 1);
    const int grp = threadIdx.x / G;
    const int64_t b = static_cast<int64_t>(block) * GROUPS + grp;
    if (b >= a.B) return;   // whole groups leave together; groups never communicate below
    const int K = a.K;
    const int R = K + 2;
    const int d4 = a.d4;
    const int d = d4 * 4;

    // lane j < R owns reference j: id, delta slot, shared flag
    int32_t id_mine = 0;
    uint32_t pos_mine = 0;
    int shared_mine = 0;
    const uint32_t ref_mine = static_cast<uint32_t>(b * R + lg);
    if (lg < R) {
        id_mine = a.ids[ref_mine];
        pos_mine = a.posbuf[ref_mine];
        shared_mine = a.refshared[ref_mine];
    }
    const int shared0 = __shfl(shared_mine, 0, G);
    const uint32_t pos0 = __shfl(pos_mine, 0, G);
    const uint32_t rank0 = shared0 ? arrival_rank<G>(a, pos0, lg) : ~0u;

    const int32_t src = __shfl(id_mine, 0, G);
    float4* xrow = a.X + static_cast<int64_t>(src) * d4;
    float4 xr[NCH];
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int ci = lg + i * G;
        xr[i] = (ci < d4) ? xrow[ci] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    float xt[4 * NCH];   // x in consecutive-dword layout, for the atomic path
    to_consecutive<G, NCH>(xr, xt, lds[grp], lg);

    float4 dx[NCH];
#pragma unroll
    for (int i = 0; i < NCH; ++i) dx[i] = make_float4(0.f, 0.f, 0.f, 0.f);

    // (lane 0's reference, the vertex row, has been ranked above)
    context_rows_of_pair<G, NCH, JB, 1>(a, K, d4, d, xr, xt, dx, id_mine, pos_mine, lg >= 1 ? shared_mine : 0, ref_mine, lg);

    if (!shared0) {
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int ci = lg + i * G;
            if (ci < d4)
                xrow[ci] = make_float4(xr[i].x + dx[i].x, xr[i].y + dx[i].y, xr[i].z + dx[i].z, xr[i].w + dx[i].w);
        }
    } else {
        shared_row_delta<G, NCH>(a, pos0, static_cast<uint32_t>(b * R), rank0, dx, lds[grp], lg, d4, xrow);
    }
}

// ---------------------------------------------------------------------------------------------
// train kernel of the walk mode: one lane group per walk position.  The source row is gathered once
// and stays in registers for the position's `window` pairs; its delta is summed over all of them
// and written once.  Each pair's K+1 context rows are handled exactly as in the pair mode.
// ---------------------------------------------------------------------------------------------
template <int G, int NCH, int JB>
__global__ __launch_bounds__(kTrainThreads) void train_walk_kernel(TrainArgs a, PrepArgs next, unsigned claim_blocks, unsigned period)
{
    constexpr int GROUPS = kTrainThreads / G;
    __shared__ float lds[GROUPS][4 * G * NCH];
    unsigned block;
    if (fused_block(claim_blocks, period, &block)) {
        if (block < next.fetch_blocks) {   // sample prefetch for the batch after the next
            fetch_pairs(next.fetch_src, next.fetch_dst, next.fetch_n, static_cast<int64_t>(block) * kTrainThreads + threadIdx.x,
                        static_cast<int64_t>(next.fetch_blocks) * kTrainThreads);
            return;
        }
        block -= next.fetch_blocks;
        for (unsigned tid = threadIdx.x; tid < 256u; tid += kTrainThreads) claim_refs(next, block, tid);
        return;
    }
    const int lg = threadIdx.x & (G - 1);
    const int grp = threadIdx.x / G;
    const int64_t p = static_cast<int64_t>(block) * GROUPS + grp;
    if (p >= a.B) return;   // whole groups leave together; groups never communicate below
    const int K = a.K;
    const int d4 = a.d4;
    const int d = d4 * 4;
    const int64_t R = 1 + static_cast<int64_t>(a.window) * (K + 1);
    const int64_t ref0 = p * R;

    const int32_t src = a.ids[ref0];
    if (src < 0) return;    // no pair starts at this position (uniform over the group)
    const uint32_t pos0 = a.posbuf[ref0];
    const int shared0 = a.refshared[ref0];
    const uint32_t rank0 = shared0 ? arrival_rank<G>(a, pos0, lg) : ~0u;

    float4* xrow = a.X + static_cast<int64_t>(src) * d4;
    float4 xr[NCH];
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int ci = lg + i * G;
        xr[i] = (ci < d4) ? xrow[ci] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    float xt[4 * NCH];   // x in consecutive-dword layout, for the atomic path
    to_consecutive<G, NCH>(xr, xt, lds[grp], lg);

    float4 dx[NCH];
#pragma unroll
    for (int i = 0; i < NCH; ++i) dx[i] = make_float4(0.f, 0.f, 0.f, 0.f);

    for (int j = 0; j < a.window; ++j) {
        // lane l <= K owns context reference l of pair j
        int32_t id_mine = -1;
        uint32_t pos_mine = 0;
        int shared_mine = 0;
        const int64_t ref = ref0 + 1 + static_cast<int64_t>(j) * (K + 1) + lg;
        if (lg <= K) {
            id_mine = a.ids[ref];
            if (id_mine >= 0) {
                pos_mine = a.posbuf[ref];
                shared_mine = a.refshared[ref];
            }
        }
        if (__shfl(id_mine, 0, G) < 0) continue;   // the walk has no pair j here; a pair's references exist together
        context_rows_of_pair<G, NCH, JB, 0>(a, K, d4, d, xr, xt, dx, id_mine, pos_mine, shared_mine, static_cast<uint32_t>(ref), lg);
    }

    if (!shared0) {
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int ci = lg + i * G;
            if (ci < d4)
                xrow[ci] = make_float4(xr[i].x + dx[i].x, xr[i].y + dx[i].y, xr[i].z + dx[i].z, xr[i].w + dx[i].w);
        }
    } else {
        shared_row_delta<G, NCH>(a, pos0, static_cast<uint32_t>(ref0), rank0, dx, lds[grp], lg, d4, xrow);
    }
}

// ---------------------------------------------------------------------------------------------
// train kernel of the walk mode by segments: one workgroup per segment of E = threads / G
// consecutive entries of a walk, one lane group per entry.  All vertex rows of the segment's entries
// and all context rows that serve as their samples' contexts (E + window - 1 of them) are gathered
// once into LDS.  Each group then plays two parts:
//   source   its entry against the up to `window` following context rows (from LDS) and against the
//            K negatives of each sample (from memory): sums dx in registers, updates the negatives;
//   context  its entry's context row (and, for the first window-1 groups, one of the rows past the
//            segment's end) against the vertex rows (from LDS) of the up to `window` preceding
//            entries of this segment: sums dc in registers.
// The positive score of a sample is therefore computed twice (both ends need its coefficient); the
// rows are what costs.  Every row is then written once: in place if no other reference names it,
// else to its slot with atomics (the context rows next to a segment boundary get contributions
// from both segments and are always of that kind).
// ---------------------------------------------------------------------------------------------
template <int G, int NCH, int JB>
__global__ __launch_bounds__(kTrainThreads) void train_seg_kernel(TrainArgs a, PrepArgs next, unsigned claim_blocks, unsigned period)
{
    constexpr int E = kTrainThreads / G;
    constexpr int ROW = 4 * G * NCH;              // floats per staged row (>= d)
    extern __shared__ float seg_lds[];
    float* scratch = seg_lds;                      // [E][ROW]        layout changes for the atomic path
    float* xs = scratch + E * ROW;                 // [E][ROW]        vertex rows of the entries
    float* cs = xs + E * ROW;                      // [E + window - 1][ROW]  context rows
    const int CT = E + a.window - 1;
    int32_t* cid = reinterpret_cast<int32_t*>(cs + CT * ROW);   // [CT] ids of the context rows (-1: absent)
    int32_t* xid = cid + CT;                                    // [E]  ids of the vertex rows (-1: absent)
    unsigned block;
    if (fused_block(claim_blocks, period, &block)) {
        if (block < next.fetch_blocks) {   // sample prefetch for the batch after the next
            fetch_pairs(next.fetch_src, next.fetch_dst, next.fetch_n, static_cast<int64_t>(block) * kTrainThreads + threadIdx.x,
                        static_cast<int64_t>(next.fetch_blocks) * kTrainThreads);
            return;
        }
        block -= next.fetch_blocks;
        for (unsigned tid = threadIdx.x; tid < 256u; tid += kTrainThreads) claim_refs(next, block, tid);
        return;
    }
    const int lg = threadIdx.x & (G - 1);
    const int grp = threadIdx.x / G;
    const int K = a.K;
    const int W = a.window;
    const int d4 = a.d4;
    const int d = d4 * 4;
    const int64_t R = E + CT + static_cast<int64_t>(E) * W * K;
    if (static_cast<int64_t>(block) >= a.B) return;             // a.B = segments of the batch (uniform over the workgroup)
    const int64_t ref0 = static_cast<int64_t>(block) * R;

    // my entry's vertex row, and the context rows grp and grp + E of the segment's list
    const int32_t src = a.ids[ref0 + grp];
    uint32_t pos_x = 0, rank_x = ~0u;
    int shared_x = 0;
    float4 xr[NCH];
#pragma unroll
    for (int i = 0; i < NCH; ++i) xr[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    float4* xrow = a.X;
    if (src >= 0) {
        pos_x = a.posbuf[ref0 + grp];
        shared_x = a.refshared[ref0 + grp];
        if (shared_x) rank_x = arrival_rank<G>(a, pos_x, lg);
        xrow = a.X + static_cast<int64_t>(src) * d4;
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int ci = lg + i * G;
            if (ci < d4) xr[i] = xrow[ci];
        }
    }
#pragma unroll
    for (int i = 0; i < NCH; ++i) reinterpret_cast<float4*>(xs + grp * ROW)[lg + i * G] = xr[i];
    if (lg == 0) xid[grp] = src;
    for (int row = grp; row < CT; row += E) {
        const int32_t id = a.ids[ref0 + E + row];
        if (lg == 0) cid[row] = id;
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int ci = lg + i * G;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (id >= 0 && ci < d4) v = (a.C + static_cast<int64_t>(id) * d4)[ci];
            reinterpret_cast<float4*>(cs + row * ROW)[ci] = v;
        }
    }
    __syncthreads();

    // ---- source part
    if (src >= 0) {
        float xt[4 * NCH];   // x in consecutive-dword layout, for the atomic path
        to_consecutive<G, NCH>(xr, xt, scratch + grp * ROW, lg);
        float4 dx[NCH];
#pragma unroll
        for (int i = 0; i < NCH; ++i) dx[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int j = 1; j <= W; ++j) {
            const int row = grp + j - 1;                      // context row of entry (mine + j)
            if (cid[row] < 0) continue;                       // no such sample (uniform over the group)
            float4 cr[NCH];
            float p = 0.0f;
#pragma unroll
            for (int i = 0; i < NCH; ++i) {
                cr[i] = reinterpret_cast<const float4*>(cs + row * ROW)[lg + i * G];
                p += dot4(xr[i], cr[i]);
            }
            p = group_sum<G>(p);
            const float g0 = a.lr * (1.0f - sigmoidf(p));
#pragma unroll
            for (int i = 0; i < NCH; ++i) dx[i] = axpy4(g0, cr[i], dx[i]);
            if (K > 0) {
                // lane k < K owns negative k of this sample
                int32_t id_mine = -1;
                uint32_t pos_mine = 0;
                int shared_mine = 0;
                const int64_t ref = ref0 + E + CT + (static_cast<int64_t>(grp) * W + (j - 1)) * K + lg;
                if (lg < K) {
                    id_mine = a.ids[ref];
                    pos_mine = a.posbuf[ref];
                    shared_mine = a.refshared[ref];
                }
                context_rows_of_pair<G, NCH, JB, 0, false>(a, K - 1, d4, d, xr, xt, dx, id_mine, pos_mine, shared_mine,
                                                           static_cast<uint32_t>(ref), lg);
            }
        }
        if (!shared_x) {
#pragma unroll
            for (int i = 0; i < NCH; ++i) {
                const int ci = lg + i * G;
                if (ci < d4)
                    xrow[ci] = make_float4(xr[i].x + dx[i].x, xr[i].y + dx[i].y, xr[i].z + dx[i].z, xr[i].w + dx[i].w);
            }
        } else {
            shared_row_delta<G, NCH>(a, pos_x, static_cast<uint32_t>(ref0 + grp), rank_x, dx, scratch + grp * ROW, lg, d4, xrow);
        }
    }

    // ---- context part: context row `row` is entry p0 + 1 + row; its sources in this segment are the
    // entries with local index max(0, row + 1 - W) .. min(row, E - 1)
    for (int row = grp; row < CT; row += E) {
        const int32_t id = cid[row];
        if (id < 0) continue;
        const int64_t ref = ref0 + E + row;
        const uint32_t pos_c = a.posbuf[ref];
        const int shared_c = a.refshared[ref];
        const uint32_t rank_c = shared_c ? arrival_rank<G>(a, pos_c, lg) : ~0u;
        float4 cr[NCH], dc[NCH];
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            cr[i] = reinterpret_cast<const float4*>(cs + row * ROW)[lg + i * G];
            dc[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
        const int lo = row + 1 - W > 0 ? row + 1 - W : 0, hi = row < E - 1 ? row : E - 1;
        for (int sl = lo; sl <= hi; ++sl) {
            if (xid[sl] < 0) continue;
            float4 xv[NCH];
            float p = 0.0f;
#pragma unroll
            for (int i = 0; i < NCH; ++i) {
                xv[i] = reinterpret_cast<const float4*>(xs + sl * ROW)[lg + i * G];
                p += dot4(xv[i], cr[i]);
            }
            p = group_sum<G>(p);
            const float g0 = a.lr * (1.0f - sigmoidf(p));
#pragma unroll
            for (int i = 0; i < NCH; ++i) dc[i] = axpy4(g0, xv[i], dc[i]);
        }
        if (!shared_c) {
            float4* crow = a.C + static_cast<int64_t>(id) * d4;
#pragma unroll
            for (int i = 0; i < NCH; ++i) {
                const int ci = lg + i * G;
                if (ci < d4)
                    crow[ci] = make_float4(cr[i].x + dc[i].x, cr[i].y + dc[i].y, cr[i].z + dc[i].z, cr[i].w + dc[i].w);
            }
        } else {
            shared_row_delta<G, NCH>(a, pos_c, static_cast<uint32_t>(ref), rank_c, dc, scratch + grp * ROW, lg, d4,
                                     a.C + static_cast<int64_t>(id) * d4);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// apply kernel.  Two kinds of blocks:
//   resolve_blocks of them (spread over the grid): resolve phase of the next batch (other set of
//                         hash state)
//   the rest              sweep the batch's hash positions in order, 8 per thread: read the shared
//                         flags, empty the positions and clear the flags with full-width stores
//                         (a linear pass is far cheaper than one partial store per reference), collect
//                         the shared rows in LDS, then 16-lane groups add each row's deltas - the
//                         buffer rows of its member list, the slot if references beyond the list
//                         used it - to the table row and zero what they used.
// ---------------------------------------------------------------------------------------------
// Positions per sweep thread are a launch choice (2, 4 or 8): fewer give the row work more workgroups,
// more make the sweep itself cheaper.  Position counts are multiples of the largest block's span.
constexpr int kSweepPerBlock = 256 * 8;

__device__ __forceinline__ float4 add4(float4 a, float4 b) { return make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w); }

struct ApplyArgs {
    float4* X;
    float4* C;
    int32_t d4;
    float4* delta;
    uint32_t positions;   // hash positions in use for this batch (a power of two, multiple of 2048)
    unsigned long long* slots;
    uint8_t* shared;
    uint32_t list_cap;    // as in TrainArgs
    uint32_t* count;
    const uint32_t* members;
    const float4* dbuf;
    int32_t direct;       // per-sample mode: the train kernel has already added the shared rows' deltas to the tables
};

template <int kSweepPerThread, int GL, int CH>
__global__ __launch_bounds__(256) void apply_kernel(ApplyArgs a, PrepArgs next, unsigned resolve_blocks,
                                                    unsigned period)
{
    constexpr int kSpan = 256 * kSweepPerThread;   // positions per workgroup
    __shared__ uint2 todo_list[kSpan];   // (position, key) of the shared rows of this block's span
    __shared__ int todo_count;
    unsigned block;
    if (fused_block(resolve_blocks, period, &block)) {
        resolve_refs(next, block);
        return;
    }
    if (threadIdx.x == 0) todo_count = 0;
    __syncthreads();
    const uint32_t first = block * kSpan + threadIdx.x * kSweepPerThread;
    using flags_t = std::conditional_t<kSweepPerThread == 8, uint64_t, std::conditional_t<kSweepPerThread == 4, uint32_t, uint16_t>>;
    static_assert(kSweepPerThread == 8 || kSweepPerThread == 4 || kSweepPerThread == 2, "flags are read as one word");
    const uint64_t flags = *reinterpret_cast<const flags_t*>(a.shared + first);
    if (flags) {
        *reinterpret_cast<flags_t*>(a.shared + first) = 0;
#pragma unroll
        for (int i = 0; i < kSweepPerThread; ++i) {
            if ((flags >> (8 * i)) & 0xFFull) {
                const uint32_t key = static_cast<uint32_t>(a.slots[first + i] >> 32);
                todo_list[atomicAdd(&todo_count, 1)] = make_uint2(first + i, key);
            }
        }
    }
    {
        ulonglong2* out = reinterpret_cast<ulonglong2*>(a.slots + first);
        const ulonglong2 empty2 = make_ulonglong2(kEmptySlot, kEmptySlot);
#pragma unroll
        for (int i = 0; i < kSweepPerThread / 2; ++i) out[i] = empty2;
    }
    __syncthreads();
    const int n = a.direct ? 0 : todo_count;
    const int lg = threadIdx.x & (GL - 1);
    for (int e = threadIdx.x / GL; e < n; e += 256 / GL) {
        const uint2 item = todo_list[e];
        float4* row = ((item.y & 0x80000000u) ? a.C : a.X) + static_cast<int64_t>(item.y & 0x7FFFFFFFu) * a.d4;
        float4* slot = a.delta + static_cast<int64_t>(item.x) * a.d4;
        // list path: the row's first arrivals left their deltas in dbuf; only later ones used the slot
        uint32_t listed = 0, member = 0;
        bool use_slot = true;
        if (a.list_cap) {
            const uint32_t arrived = a.count[item.x];
            // (entries past the list's end hold stale indices; they are not used)
            if (static_cast<uint32_t>(lg) < kListCap) member = a.members[static_cast<int64_t>(item.x) * kListCap + lg];
            listed = arrived < a.list_cap ? arrived : a.list_cap;
            use_slot = arrived > listed;
            if (lg == 0) a.count[item.x] = 0u;
        }
        // CH chunks of a row per lane and pass, all of a pass's loads issued before its stores (a
        // 2 KB row in passes of 2 chunks would pay four dependent round trips instead of one)
        for (int c0 = 0; c0 < a.d4; c0 += GL * CH) {
            float4 acc[CH];
            bool valid[CH];
#pragma unroll
            for (int i = 0; i < CH; ++i) {
                const int ci = c0 + lg + GL * i;
                valid[i] = ci < a.d4;
                acc[i] = valid[i] ? row[ci] : make_float4(0.f, 0.f, 0.f, 0.f);
            }
            if (use_slot) {
                float4 sv[CH];
#pragma unroll
                for (int i = 0; i < CH; ++i) sv[i] = valid[i] ? slot[c0 + lg + GL * i] : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                for (int i = 0; i < CH; ++i) acc[i] = add4(acc[i], sv[i]);
            }
            // the list's buffer rows, MB members' loads in flight together
            constexpr uint32_t MB = CH >= 16 ? 1 : (16 / CH < kListCap ? 16 / CH : kListCap);
            for (uint32_t r0 = 0; r0 < listed; r0 += MB) {
                float4 dv[MB][CH];
#pragma unroll
                for (uint32_t r = 0; r < MB; ++r) {
                    const float4* src = a.dbuf + static_cast<int64_t>(__shfl(member, static_cast<int>((r0 + r) & (kListCap - 1)), GL)) * a.d4;
#pragma unroll
                    for (int i = 0; i < CH; ++i)
                        dv[r][i] = (r0 + r < listed && valid[i]) ? src[c0 + lg + GL * i] : make_float4(0.f, 0.f, 0.f, 0.f);
                }
#pragma unroll
                for (uint32_t r = 0; r < MB; ++r)
#pragma unroll
                    for (int i = 0; i < CH; ++i) acc[i] = add4(acc[i], dv[r][i]);
            }
#pragma unroll
            for (int i = 0; i < CH; ++i)
                if (valid[i]) row[c0 + lg + GL * i] = acc[i];
            if (use_slot) {
#pragma unroll
                for (int i = 0; i < CH; ++i)
                    if (valid[i]) slot[c0 + lg + GL * i] = make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// loss kernel (ne_eval_loss): sampling + scoring fused, tables read-only.
// ---------------------------------------------------------------------------------------------
struct LossArgs {
    const float4* X;
    const float4* C;
    const int2* pairs;
    int64_t B;
    int32_t K;
    int32_t d4;
    uint64_t sample_base;
    uint32_t k0, k1;
    const uint2* alias;
    uint64_t alias_n;
    int32_t alias_base;
    int32_t* neg_out;
    double* loss;
};

template <int G, int NCH, int JB>
__global__ __launch_bounds__(256) void loss_kernel(LossArgs a)
{
    constexpr int GROUPS = 256 / G;
    const int lg = threadIdx.x & (G - 1);
    const int64_t b_raw = static_cast<int64_t>(blockIdx.x) * GROUPS + (threadIdx.x / G);
    const bool active = b_raw < a.B;
    const int64_t b = active ? b_raw : a.B - 1;
    const int K = a.K;
    const int d4 = a.d4;
    const int2 pr = a.pairs[b];

    // lane lg owns context row j = lg of the pair: j = 0 the positive, j = 1..K negative j-1
    int32_t id_mine = pr.y;
    if (lg >= 1 && lg <= K) {
        id_mine = draw_negative(a.sample_base + static_cast<uint64_t>(b), static_cast<uint32_t>(lg - 1), a.k0, a.k1,
                                a.alias, a.alias_n, a.alias_base);
        if (active && a.neg_out) a.neg_out[b * K + (lg - 1)] = id_mine;
    }
    float4 xr[NCH];
    const float4* xrow = a.X + static_cast<int64_t>(pr.x) * d4;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int ci = lg + i * G;
        xr[i] = (ci < d4) ? xrow[ci] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    float term_mine = 0.0f;   // lane j keeps the loss term of row j
    for (int j0 = 0; j0 <= K; j0 += JB) {
        float part[JB];
#pragma unroll
        for (int jj = 0; jj < JB; ++jj) {
            const int j = j0 + jj;
            const int32_t id = __shfl(id_mine, j <= K ? j : K, G);
            const float4* crow = a.C + static_cast<int64_t>(id) * d4;
            float p = 0.0f;
#pragma unroll
            for (int i = 0; i < NCH; ++i) {
                const int ci = lg + i * G;
                if (j <= K && ci < d4) p += dot4(xr[i], crow[ci]);
            }
            part[jj] = p;
        }
#pragma unroll
        for (int jj = 0; jj < JB; ++jj) part[jj] = group_sum<G>(part[jj]);
#pragma unroll
        for (int jj = 0; jj < JB; ++jj) {
            const int j = j0 + jj;
            if (j <= K && lg == j) term_mine = softplusf(j == 0 ? -part[jj] : part[jj]);
        }
    }
    float l = (active && lg <= K) ? term_mine : 0.0f;
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
// score kernel (ne_score_pairs): the model's similarity score of arbitrary node pairs, for
// evaluation (link prediction, Sec. V-B).  16 lanes per pair, float4 chunks strided over the row.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void score_pairs_kernel(const float4* __restrict__ A, const float4* __restrict__ Bt,
                                                          const int2* __restrict__ pairs, int64_t n, int32_t d4,
                                                          float* __restrict__ scores)
{
    const int lg = threadIdx.x & 15;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * 16;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * 16 + (threadIdx.x >> 4); i < n; i += stride) {
        const int2 pr = pairs[i];
        const float4* a = A + static_cast<int64_t>(pr.x) * d4;
        const float4* b = Bt + static_cast<int64_t>(pr.y) * d4;
        float p = 0.0f;
        for (int c = lg; c < d4; c += 16) p += dot4(a[c], b[c]);
        p = group_sum<16>(p);
        if (lg == 0) scores[i] = p;
    }
}

// ---------------------------------------------------------------------------------------------
// launch-shape selection
// ---------------------------------------------------------------------------------------------
struct Shape { int G, NCH; };

// Smallest lane group that covers dim/4 float4 chunks and has a lane for each of the K+2 references.
bool pick_shape(int32_t d4, int32_t K, Shape* out)
{
    // one float4 per lane as long as a wavefront holds the row: measured 4-5 % faster at dim 128 than 16 lanes x 2
    static const Shape order[] = {{8, 1}, {16, 1}, {32, 1}, {64, 1}, {64, 2}, {64, 4}};
    for (const Shape& s : order) {
        if (s.G * s.NCH >= d4 && s.G >= K + 2) { *out = s; return true; }
    }
    return false;
}

#define NE_FOR_EACH_SHAPE(M) M(8, 1) M(16, 1) M(32, 1) M(64, 1) M(64, 2) M(64, 4)

hipError_t launch_train(const Shape& s, const TrainArgs& a, const PrepArgs& next, hipStream_t st)
{
    const int groups = kTrainThreads / s.G;
    const unsigned claim_blocks = prep_blocks(next.refs) + next.fetch_blocks;   // helper workgroups
    const unsigned grid = claim_blocks + static_cast<unsigned>((a.B + groups - 1) / groups);
    const unsigned period = claim_blocks ? grid / claim_blocks : 1u;
    // context rows gathered together per lane group: 2 measured +1.3 % over 6 at dim 128 (fewer registers,
    // more wavefronts resident; the kernel is bound by throughput, not by one group's latency), except with
    // the list path, where 6 is 1.5 % ahead
    const bool few = a.list_cap == 0;
#define NE_CASE(G_, N_)                                                                          \
    if (s.G == G_ && s.NCH == N_) {                                                              \
        if (few) hipLaunchKernelGGL((train_kernel<G_, N_, 2>), dim3(grid), dim3(kTrainThreads), 0, st, a, next, claim_blocks, period); \
        else hipLaunchKernelGGL((train_kernel<G_, N_, 6>), dim3(grid), dim3(kTrainThreads), 0, st, a, next, claim_blocks, period); \
        return hipGetLastError();                                                                \
    }
    NE_FOR_EACH_SHAPE(NE_CASE)
#undef NE_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_train_walk(const Shape& s, const TrainArgs& a, const PrepArgs& next, hipStream_t st)
{
    const int groups = kTrainThreads / s.G;
    const unsigned claim_blocks = prep_blocks(next.refs) + next.fetch_blocks;   // helper workgroups
    const unsigned grid = claim_blocks + static_cast<unsigned>((a.B + groups - 1) / groups);
    const unsigned period = claim_blocks ? grid / claim_blocks : 1u;
#define NE_CASE(G_, N_)                                                                          \
    if (s.G == G_ && s.NCH == N_) {                                                              \
        hipLaunchKernelGGL((train_walk_kernel<G_, N_, 6>), dim3(grid), dim3(kTrainThreads), 0, st, a, next, claim_blocks, period); \
        return hipGetLastError();                                                                \
    }
    NE_FOR_EACH_SHAPE(NE_CASE)
#undef NE_CASE
    return hipErrorInvalidValue;
}

// LDS of the segment kernel: scratch, vertex rows and context rows of a segment, and their ids
size_t seg_lds_bytes(const Shape& s, int window)
{
    const size_t E = kTrainThreads / s.G, row = 4 * static_cast<size_t>(s.G) * s.NCH, CT = E + window - 1;
    return (2 * E + CT) * row * 4 + (CT + E) * 4;
}

hipError_t launch_train_seg(const Shape& s, const TrainArgs& a, const PrepArgs& next, unsigned segments, hipStream_t st)
{
    const unsigned claim_blocks = prep_blocks(next.refs) + next.fetch_blocks;   // helper workgroups
    const unsigned grid = claim_blocks + segments;
    const unsigned period = claim_blocks ? grid / claim_blocks : 1u;
    const size_t lds = seg_lds_bytes(s, a.window);
#define NE_CASE(G_, N_)                                                                          \
    if (s.G == G_ && s.NCH == N_) {                                                              \
        hipLaunchKernelGGL((train_seg_kernel<G_, N_, 6>), dim3(grid), dim3(kTrainThreads), lds, st, a, next, claim_blocks, period); \
        return hipGetLastError();                                                                \
    }
    NE_FOR_EACH_SHAPE(NE_CASE)
#undef NE_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_loss(const Shape& s, const LossArgs& a, hipStream_t st)
{
    const int groups = 256 / s.G;
    const unsigned grid = static_cast<unsigned>((a.B + groups - 1) / groups);
#define NE_CASE(G_, N_)                                                                          \
    if (s.G == G_ && s.NCH == N_) {                                                              \
        hipLaunchKernelGGL((loss_kernel<G_, N_, 6>), dim3(grid), dim3(256), 0, st, a);           \
        return hipGetLastError();                                                                \
    }
    NE_FOR_EACH_SHAPE(NE_CASE)
#undef NE_CASE
    return hipErrorInvalidValue;
}

// Largest batch: keeps every grid and the hash capacity inside 32 bits.
constexpr int64_t kMaxBatch = static_cast<int64_t>(1) << 22;
// Hash positions per reference, before rounding up to a power of two (load <= 1/2).  Four per
// reference mean less probing but a longer sweep and twice the footprint of the delta slots, and
// measured slower at every size tried (100 M nodes x dim 128: -1.6 %, 20 M x 512: -6 %, 1 M x 128: -7 %);
// eight: -12 %.
constexpr uint32_t kHashFactor = 2;
// helper workgroups that prefetch the samples of a later batch from pinned host memory (512 KB per batch of 65536)
constexpr unsigned kFetchBlocks = 8;

// How a batch treats its shared rows.  Tables that are small next to the batch make most references name
// shared rows: the train kernel is then bound by the atomics' rate, and the list path (plain stores per
// reference, summed by the apply kernel) pays: +20 % at 1 M nodes x dim 128 with 458 752 references per
// batch.  Where the atomics hide behind the row traffic it costs 4-12 %.  Break-even, measured on R-MAT
// pairs as nodes per reference: 20 at dim 32, 12 at dim 128, 8 at dim 256, 4 at dim 512 (K = 10); the
// rule below stays a little under it.  The sweep gives each thread 4 positions (2 with the list path,
// whose row work is longer): 8 made the sweep cheaper but left the row work too few workgroups (-3.6 %).
// ne_set_tuning overrides both.
struct BatchTuning { uint32_t list_cap; int sweep_per_thread; };
inline BatchTuning batch_tuning(const ne_tables* t, uint32_t refs)
{
    const int64_t per_ref = 1500 / t->dim < 20 ? 1500 / t->dim : 20;   // nodes per reference up to which lists pay
    const bool small_tables = t->num_nodes <= per_ref * static_cast<int64_t>(refs);
    BatchTuning b;
    b.list_cap = t->tune_list_cap >= 0 ? static_cast<uint32_t>(t->tune_list_cap) : (small_tables ? kListCap : 0u);
    b.sweep_per_thread = t->tune_sweep > 0 ? t->tune_sweep : (small_tables ? 2 : 4);
    return b;
}

bool workspace_layout(int32_t dim, int64_t max_B, int32_t max_K, char* base, Workspace* w)
{
    if (dim < 4 || dim > NE_MAX_DIM || dim % 4 != 0 || max_B < 1 || max_B > kMaxBatch || max_K < 0 ||
        max_K > NE_MAX_NEGATIVES)
        return false;
    const uint64_t refs = static_cast<uint64_t>(max_B) * (max_K + 2);
    uint64_t cap = 2048;   // one sweep block of the apply kernel
    while (cap < kHashFactor * refs) cap <<= 1;
    auto up = [](size_t v) { return (v + 255) & ~static_cast<size_t>(255); };
    size_t off = 0;
    auto take = [&](size_t bytes) { char* p = base + off; off = up(off + bytes); return p; };
    w->cap = static_cast<uint32_t>(cap);
    for (int i = 0; i < 2; ++i) {
        w->prep[i].slots = reinterpret_cast<unsigned long long*>(take(cap * 8));
        w->prep[i].shared = reinterpret_cast<uint8_t*>(take(cap));
        w->prep[i].ids = reinterpret_cast<int32_t*>(take(refs * 4));
        w->prep[i].posbuf = reinterpret_cast<uint32_t*>(take(refs * 4));
        w->prep[i].refshared = reinterpret_cast<uint8_t*>(take(refs));
    }
    w->delta = reinterpret_cast<float*>(take(cap * static_cast<size_t>(dim) * 4));
    w->count = reinterpret_cast<uint32_t*>(take(cap * 4));
    w->members = reinterpret_cast<uint32_t*>(take(cap * static_cast<size_t>(kListCap) * 4));
    w->dbuf = reinterpret_cast<float*>(take(refs * static_cast<size_t>(dim) * 4));
    w->total_bytes = off;
    return true;
}

hipError_t launch_fill(uint32_t* p, size_t n, uint32_t v, hipStream_t st)
{
    if (n == 0) return hipSuccess;
    const size_t want = (n + 255) / 256;
    const unsigned grid = static_cast<unsigned>(want < 16384 ? want : 16384);
    hipLaunchKernelGGL(fill_u32_kernel, dim3(grid), dim3(256), 0, st, p, n, v);
    return hipGetLastError();
}

// The state every batch expects to find: hash positions empty, flags, delta slots and arrival counters zero.
hipError_t clear_workspace(const Workspace& w, int32_t dim, hipStream_t st)
{
    hipError_t e = hipSuccess;
    for (int i = 0; i < 2 && e == hipSuccess; ++i) {
        e = launch_fill(reinterpret_cast<uint32_t*>(w.prep[i].slots), static_cast<size_t>(w.cap) * 2, 0xFFFFFFFFu, st);
        if (e == hipSuccess) e = launch_fill(reinterpret_cast<uint32_t*>(w.prep[i].shared), w.cap / 4, 0u, st);
    }
    if (e == hipSuccess) e = launch_fill(reinterpret_cast<uint32_t*>(w.delta), static_cast<size_t>(w.cap) * dim, 0u, st);
    if (e == hipSuccess) e = launch_fill(w.count, w.cap, 0u, st);
    return e;
}

ne_status check_batch_args(const ne_tables* t, const ne_alias* al, const int32_t* pairs, int64_t B, int32_t K,
                           Shape* shape)
{
    if (!t) return fail(NE_ERR_ARG, "tables handle is NULL");
    if (B < 0 || B > kMaxBatch) return fail(NE_ERR_ARG, "B out of range [0, 2^22]");
    if (K < 0 || K > NE_MAX_NEGATIVES) return fail(NE_ERR_ARG, "K out of range [0, 62]");
    if (K > 0 && !al) return fail(NE_ERR_ARG, "alias handle is NULL but K > 0");
    if (B > 0 && !pairs) return fail(NE_ERR_ARG, "pairs_dev is NULL");
    if (!aligned(pairs, 8)) return fail(NE_ERR_ARG, "pairs_dev must be 8-byte aligned");
    if (al && (al->base < 0 || al->base + al->n > t->num_nodes))
        return fail(NE_ERR_STATE, "alias id range [base, base+n) is not inside the tables' [0, num_nodes)");
    if (!pick_shape(t->dim / 4, K, shape)) return fail(NE_ERR_ARG, "no launch shape for this (dim, K)");
    return NE_OK;
}

// The launches of a run of batches, common to the pair and the walk shapes: claim and resolve of the
// first batch stand alone; then per batch kernel A = train(i) + claim(i+1) (+ sample prefetch) and
// kernel B = apply(i) + resolve(i+1).  prep(i) describes batch i (refs = 0 past the end); train(ta, next)
// launches the shape's train kernel.
template <class PrepFn, class TrainFn>
ne_status run_batches(ne_tables* t, int64_t n_batches, int64_t R, int32_t window, int32_t K, const float* lr_host,
                             hipStream_t st, PrepFn prep, TrainFn train, bool direct = false)
{
    const Workspace& w = t->ws;
    // A launch that failed part-way through an earlier run left hash positions, flags or slots in use:
    // start from a clean workspace again (the tables may hold a partly applied batch; that is the caller's
    // to judge from the error it got then).
    if (t->workspace_dirty) {
        const hipError_t ce = clear_workspace(w, t->dim, st);
        if (ce != hipSuccess) return fail(NE_ERR_HIP, std::string("workspace re-clear launch: ") + hipGetErrorString(ce));
        t->workspace_dirty = false;
    }
    t->workspace_dirty = true;   // until the last launch of this run has been enqueued
    PrepArgs cur = prep(0);
    cur.fetch_blocks = 0;   // a prefetch only rides in train launches
    const unsigned grid0 = prep_blocks(cur.refs);
    hipLaunchKernelGGL(claim_kernel, dim3(grid0), dim3(256), 0, st, cur);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(NE_ERR_HIP, std::string("claim launch: ") + hipGetErrorString(e));
    hipLaunchKernelGGL(resolve_kernel, dim3(grid0), dim3(256), 0, st, cur);
    e = hipGetLastError();
    if (e != hipSuccess) return fail(NE_ERR_HIP, std::string("resolve launch: ") + hipGetErrorString(e));

    for (int64_t i = 0; i < n_batches; ++i) {
        const PrepArgs next = prep(i + 1);
        const PrepSlot& ps = w.prep[i & 1];
        TrainArgs ta{};
        ta.X = reinterpret_cast<float4*>(t->vertex); ta.C = reinterpret_cast<float4*>(t->context);
        ta.B = cur.refs / R; ta.window = window; ta.K = K; ta.d4 = t->dim / 4; ta.lr = lr_host[i];
        ta.ids = ps.ids; ta.posbuf = ps.posbuf; ta.refshared = ps.refshared; ta.delta = w.delta;
        BatchTuning tune = batch_tuning(t, cur.refs);
        if (direct) tune.list_cap = 0;   // no slots, no lists: shared rows take their atomics on the table itself
        ta.direct = direct ? 1 : 0;
        ta.list_cap = tune.list_cap; ta.count = w.count; ta.members = w.members; ta.dbuf = reinterpret_cast<float4*>(w.dbuf);
        const bool timed = profile_begin(t, st);
        e = train(ta, next);
        if (e != hipSuccess) return fail(NE_ERR_HIP, std::string("train launch: ") + hipGetErrorString(e));
        if (timed) profile_end(t, st);

        ApplyArgs aa{};
        aa.X = ta.X; aa.C = ta.C; aa.d4 = ta.d4; aa.delta = reinterpret_cast<float4*>(w.delta);
        aa.positions = cur.mask + 1; aa.slots = ps.slots; aa.shared = ps.shared;
        aa.list_cap = ta.list_cap; aa.count = w.count; aa.members = w.members; aa.dbuf = ta.dbuf; aa.direct = ta.direct;
        const unsigned resolve_blocks = prep_blocks(next.refs);
        const int per_thread = tune.sweep_per_thread;
        const unsigned sweep_blocks = aa.positions / (256u * per_thread);
        const unsigned apply_grid = resolve_blocks + sweep_blocks;
        const unsigned period = resolve_blocks ? apply_grid / resolve_blocks : 1u;
        // Row work of the apply kernel: GL lanes per row, CH dwordx4 chunks per lane and pass.  One chunk per
        // lane where a row has 32 or more (as in the train kernel; +1.1 % at dim 128), except with the list
        // path, whose passes keep several buffer rows in flight (16 lanes measured +1.8 % there); rows of more
        // than 2 chunks per lane go in passes of 8 (+1 % at dim 512).
        const bool wide = aa.d4 > 32, lanes32 = aa.d4 >= 32 && aa.list_cap == 0;
#define NE_APPLY(S_, G_, C_) hipLaunchKernelGGL((apply_kernel<S_, G_, C_>), dim3(apply_grid), dim3(256), 0, st, aa, next, resolve_blocks, period)
#define NE_APPLY_SHAPE(S_)                                                                        \
    do {                                                                                          \
        if (lanes32) { if (wide) NE_APPLY(S_, 32, 8); else NE_APPLY(S_, 32, 1); }                 \
        else { if (wide) NE_APPLY(S_, 16, 8); else NE_APPLY(S_, 16, 2); }                         \
    } while (0)
        if (per_thread == 2) NE_APPLY_SHAPE(2);
        else if (per_thread == 4) NE_APPLY_SHAPE(4);
        else NE_APPLY_SHAPE(8);
#undef NE_APPLY_SHAPE
#undef NE_APPLY
        e = hipGetLastError();
        if (e != hipSuccess) return fail(NE_ERR_HIP, std::string("apply launch: ") + hipGetErrorString(e));
        t->batches_done += 1;
        cur = next;
    }
    t->workspace_dirty = false;
    return NE_OK;
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// C ABI
// ---------------------------------------------------------------------------------------------
extern "C" {

const char* ne_last_error(void) { return g_last_error.c_str(); }

size_t ne_workspace_bytes(int32_t dim, int64_t max_batch, int32_t max_negatives)
{
    Workspace w;
    if (!workspace_layout(dim, max_batch, max_negatives, nullptr, &w)) return 0;
    return w.total_bytes;
}

ne_status ne_create_tables(ne_tables** out, int64_t num_nodes, int32_t dim, float* vertex_dev,
                           float* context_dev, uint64_t seed, int32_t init, int64_t max_batch,
                           int32_t max_negatives, void* workspace_dev, size_t workspace_bytes,
                           void* hip_stream)
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
    ne_tables* t = new (std::nothrow) ne_tables{};
    if (!t) return fail(NE_ERR_NOMEM, "host allocation failed");
    t->num_nodes = num_nodes; t->dim = dim; t->vertex = vertex_dev; t->context = context_dev; t->seed = seed;
    t->max_batch = 0; t->max_negatives = 0; t->batches_done = 0; t->workspace_dirty = false; t->profile_every = 0; t->ev_used = 0;
    t->tune_list_cap = -1; t->tune_sweep = 0;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);

    if (workspace_dev || max_batch > 0) {   // training requested
        Workspace w;
        if (!workspace_layout(dim, max_batch, max_negatives, static_cast<char*>(workspace_dev), &w)) {
            delete t;
            return fail(NE_ERR_ARG, "max_batch must be in [1, 2^22] and max_negatives in [0, 62]");
        }
        if (!workspace_dev || !aligned(workspace_dev, 256) || workspace_bytes < w.total_bytes) {
            delete t;
            return fail(NE_ERR_ARG, "workspace_dev is NULL, not 256-byte aligned, or smaller than ne_workspace_bytes()");
        }
        t->ws = w; t->max_batch = max_batch; t->max_negatives = max_negatives;
        const hipError_t e = clear_workspace(w, dim, st);
        if (e != hipSuccess) {
            delete t;
            return fail(NE_ERR_HIP, std::string("workspace init launch: ") + hipGetErrorString(e));
        }
    }
    if (init) {
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

void ne_destroy_tables(ne_tables* t)
{
    if (!t) return;
    for (hipEvent_t e : t->ev_zero) (void)hipEventDestroy(e);
    for (hipEvent_t e : t->ev_start) (void)hipEventDestroy(e);
    for (hipEvent_t e : t->ev_stop) (void)hipEventDestroy(e);
    delete t;
}

ne_status ne_profile_enable(ne_tables* t, int32_t every_n, int32_t max_samples)
{
    if (!t) return fail(NE_ERR_ARG, "tables handle is NULL");
    if (every_n < 0 || max_samples < 0 || max_samples > 65536) return fail(NE_ERR_ARG, "every_n or max_samples out of range");
    t->profile_every = every_n;
    t->ev_used = 0;
    while (every_n > 0 && t->ev_start.size() < static_cast<size_t>(max_samples)) {
        hipEvent_t z = nullptr, a = nullptr, b = nullptr;
        hipError_t e = hipEventCreate(&z);
        if (e == hipSuccess) e = hipEventCreate(&a);
        if (e == hipSuccess) e = hipEventCreate(&b);
        if (e != hipSuccess) {
            if (z) (void)hipEventDestroy(z);
            if (a) (void)hipEventDestroy(a);
            return fail(NE_ERR_HIP, std::string("hipEventCreate: ") + hipGetErrorString(e));
        }
        t->ev_zero.push_back(z);
        t->ev_start.push_back(a);
        t->ev_stop.push_back(b);
    }
    return NE_OK;
}

ne_status ne_profile_read(ne_tables* t, double* total_ms_host, int64_t* samples_host)
{
    if (!t || !total_ms_host || !samples_host) return fail(NE_ERR_ARG, "NULL argument");
    double total = 0.0;
    for (size_t i = 0; i < t->ev_used; ++i) {
        NE_HIP_CHECK(hipEventSynchronize(t->ev_stop[i]));
        float ms = 0.0f, overhead = 0.0f;
        NE_HIP_CHECK(hipEventElapsedTime(&ms, t->ev_start[i], t->ev_stop[i]));
        NE_HIP_CHECK(hipEventElapsedTime(&overhead, t->ev_zero[i], t->ev_start[i]));
        total += static_cast<double>(ms > overhead ? ms - overhead : 0.0f);
    }
    *total_ms_host = total;
    *samples_host = static_cast<int64_t>(t->ev_used);
    t->ev_used = 0;
    return NE_OK;
}
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

// The batches of a sequence of runs (each run: one sample block with its negative-sampling table), B pairs
// each but for the last of a run.  With staging != nullptr (one run only) pairs_dev is the device address of
// samples in pinned host memory, which are prefetched batch by batch into the ring staging[3][B].
static ne_status train_runs_impl(ne_tables* t, const ne_run* runs, int64_t n_runs, int64_t B, int32_t K,
                                 const float* lr_host, int2* staging, void* hip_stream, bool direct = false)
{
    if (!t) return fail(NE_ERR_ARG, "tables handle is NULL");
    if (n_runs < 0 || n_runs > (static_cast<int64_t>(1) << 24)) return fail(NE_ERR_ARG, "n_runs out of range");
    if (n_runs > 0 && !runs) return fail(NE_ERR_ARG, "runs_host is NULL");
    Shape shape;
    struct Batch { int64_t run, first, count; };
    std::vector<Batch> batches;
    for (int64_t r = 0; r < n_runs; ++r) {
        const ne_run& run = runs[r];
        if (run.n_pairs < 0 || run.n_pairs > (static_cast<int64_t>(1) << 40)) return fail(NE_ERR_ARG, "n_pairs out of range");
        // (an empty run may come without a pairs pointer)
        const ne_status rc = check_batch_args(t, run.alias, run.pairs_dev, run.n_pairs > 0 ? B : (B < 0 ? B : 0), K, &shape);
        if (rc != NE_OK) return rc;
        if (run.n_pairs == 0) continue;
        if (B < 1) return fail(NE_ERR_ARG, "B must be at least 1");
        if (!run.pairs_dev) return fail(NE_ERR_ARG, "pairs_dev is NULL");
        try {
            for (int64_t first = 0; first < run.n_pairs; first += B)
                batches.push_back({r, first, run.n_pairs - first < B ? run.n_pairs - first : B});
        } catch (const std::bad_alloc&) {
            return fail(NE_ERR_NOMEM, "host allocation failed");
        }
    }
    const int64_t n_batches = static_cast<int64_t>(batches.size());
    if (n_batches == 0) return NE_OK;
    if (!lr_host) return fail(NE_ERR_ARG, "lr_host is NULL");
    for (int64_t i = 0; i < n_batches; ++i)
        if (!std::isfinite(lr_host[i])) return fail(NE_ERR_ARG, "lr is not finite");
    if (t->max_batch <= 0) return fail(NE_ERR_STATE, "tables were created without a training workspace");
    if (B > t->max_batch || K > t->max_negatives)
        return fail(NE_ERR_ARG, "B or K exceeds the max_batch / max_negatives the workspace was sized for");

    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const Workspace& w = t->ws;
    const int R = K + 2;

    auto prep_args = [&](int64_t i) {
        PrepArgs pa{};
        if (i >= n_batches) return pa;   // refs = 0: nothing to prepare
        const Batch& bt = batches[i];
        const ne_run& run = runs[bt.run];
        const ne_alias* al = run.alias;
        const PrepSlot& ps = w.prep[i & 1];
        pa.pairs = staging ? staging + (i % 3) * B : reinterpret_cast<const int2*>(run.pairs_dev) + bt.first;
        if (staging && i + 1 < n_batches) {
            // the launch that trains batch i - 1 and claims batch i also fetches batch i + 1
            pa.fetch_src = reinterpret_cast<const int2*>(run.pairs_dev) + batches[i + 1].first;
            pa.fetch_dst = staging + ((i + 1) % 3) * B;
            pa.fetch_n = batches[i + 1].count;
            pa.fetch_blocks = kFetchBlocks;
        }
        pa.refs = static_cast<uint32_t>(bt.count * R); pa.R = static_cast<uint32_t>(R); pa.xrefs = 1; pa.K = K;
        pa.sample_base = run.sample_base + static_cast<uint64_t>(bt.first);
        pa.k0 = static_cast<uint32_t>(t->seed); pa.k1 = static_cast<uint32_t>(t->seed >> 32);
        pa.alias = al ? al->table : nullptr; pa.alias_n = al ? static_cast<uint64_t>(al->n) : 1; pa.alias_base = al ? al->base : 0;
        uint32_t positions = kSweepPerBlock;     // hash positions this batch uses
        while (positions < kHashFactor * static_cast<uint32_t>(bt.count * R)) positions <<= 1;
        pa.slots = ps.slots; pa.mask = positions - 1; pa.shared = ps.shared; pa.refshared = ps.refshared; pa.ids = ps.ids; pa.posbuf = ps.posbuf;
        pa.neg_out = run.neg_out_dev ? run.neg_out_dev + bt.first * K : nullptr;
        return pa;
    };

    if (staging) {   // batches 0 and 1 have no launch to ride along with
        for (int64_t i = 0; i < 2 && i < n_batches; ++i) {
            hipLaunchKernelGGL(fetch_pairs_kernel, dim3(kFetchBlocks), dim3(256), 0, st,
                               reinterpret_cast<const int2*>(runs[0].pairs_dev) + batches[i].first, staging + (i % 3) * B, batches[i].count);
            hipError_t fe = hipGetLastError();
            if (fe != hipSuccess) return fail(NE_ERR_HIP, std::string("fetch launch: ") + hipGetErrorString(fe));
        }
    }
    return run_batches(t, n_batches, R, 0, K, lr_host, st, prep_args,
                       [&](const TrainArgs& ta, const PrepArgs& next) { return launch_train(shape, ta, next, st); }, direct);
}

ne_status ne_train_runs(ne_tables* t, const ne_run* runs_host, int64_t n_runs, int64_t B, int32_t K,
                        const float* lr_host, void* hip_stream)
{
    return train_runs_impl(t, runs_host, n_runs, B, K, lr_host, nullptr, hip_stream);
}

ne_status ne_train_block(ne_tables* t, const ne_alias* al, const int32_t* pairs_dev, int64_t n_pairs, int64_t B,
                         int32_t K, const float* lr_host, uint64_t sample_base, int32_t* neg_out_dev,
                         void* hip_stream)
{
    const ne_run run{al, pairs_dev, n_pairs, sample_base, neg_out_dev};
    return train_runs_impl(t, &run, 1, B, K, lr_host, nullptr, hip_stream);
}

ne_status ne_train_block_pinned(ne_tables* t, const ne_alias* al, const int32_t* pairs_host_pinned, int64_t n_pairs,
                                int64_t B, int32_t K, const float* lr_host, uint64_t sample_base, int32_t* staging_dev,
                                int32_t* neg_out_dev, void* hip_stream)
{
    if (n_pairs > 0 && B >= 1) {
        if (!pairs_host_pinned || !aligned(pairs_host_pinned, 8)) return fail(NE_ERR_ARG, "pairs_host_pinned is NULL or not 8-byte aligned");
        if (!staging_dev || !aligned(staging_dev, 16)) return fail(NE_ERR_ARG, "staging_dev is NULL or not 16-byte aligned");
    }
    void* src_dev = const_cast<int32_t*>(pairs_host_pinned);
    if (pairs_host_pinned) {
        hipError_t e = hipHostGetDevicePointer(&src_dev, const_cast<int32_t*>(pairs_host_pinned), 0);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            return fail(NE_ERR_ARG, std::string("pairs_host_pinned is not pinned (page-locked) host memory: ") + hipGetErrorString(e));
        }
    }
    const ne_run run{al, static_cast<const int32_t*>(src_dev), n_pairs, sample_base, neg_out_dev};
    return train_runs_impl(t, &run, 1, B, K, lr_host, reinterpret_cast<int2*>(staging_dev), hip_stream);
}

ne_status ne_train_walks(ne_tables* t, const ne_alias* al, const int32_t* walks_dev, int64_t n_walks,
                         int64_t walks_per_batch, int32_t walk_len, int32_t window, int32_t K, const float* lr_host,
                         uint64_t sample_base, int32_t* neg_out_dev, void* hip_stream)
{
    if (!t) return fail(NE_ERR_ARG, "tables handle is NULL");
    if (K < 0 || K > NE_MAX_NEGATIVES) return fail(NE_ERR_ARG, "K out of range [0, 62]");
    if (K > 0 && !al) return fail(NE_ERR_ARG, "alias handle is NULL but K > 0");
    if (walk_len < 2 || walk_len > 65536) return fail(NE_ERR_ARG, "walk_len out of range [2, 65536]");
    if (window < 1 || window > 64) return fail(NE_ERR_ARG, "window out of range [1, 64]");
    if (n_walks < 0 || n_walks > (static_cast<int64_t>(1) << 32)) return fail(NE_ERR_ARG, "n_walks out of range");
    if (al && (al->base < 0 || al->base + al->n > t->num_nodes))
        return fail(NE_ERR_STATE, "alias id range [base, base+n) is not inside the tables' [0, num_nodes)");
    Shape shape;
    if (!pick_shape(t->dim / 4, K, &shape)) return fail(NE_ERR_ARG, "no launch shape for this (dim, K)");
    if (n_walks == 0) return NE_OK;
    if (!walks_dev || !aligned(walks_dev, 4)) return fail(NE_ERR_ARG, "walks_dev is NULL or misaligned");
    if (walks_per_batch < 1) return fail(NE_ERR_ARG, "walks_per_batch must be at least 1");
    if (!lr_host) return fail(NE_ERR_ARG, "lr_host is NULL");
    const int64_t n_batches = (n_walks + walks_per_batch - 1) / walks_per_batch;
    for (int64_t i = 0; i < n_batches; ++i)
        if (!std::isfinite(lr_host[i])) return fail(NE_ERR_ARG, "lr is not finite");
    if (t->max_batch <= 0) return fail(NE_ERR_STATE, "tables were created without a training workspace");
    // the workspace was sized in row references: max_batch * (max_negatives + 2)
    const int64_t R_entry = 1 + static_cast<int64_t>(window) * (K + 1);
    const int64_t ref_budget = t->max_batch * (static_cast<int64_t>(t->max_negatives) + 2);
    const int64_t wpb = walks_per_batch < n_walks ? walks_per_batch : n_walks;
    if (wpb * walk_len > ref_budget / R_entry)
        return fail(NE_ERR_ARG, "a batch of walks names more rows than the workspace was sized for: need walks_per_batch * "
                                "walk_len * (1 + window * (K + 1)) <= max_batch * (max_negatives + 2)");
    // One workgroup per segment of E consecutive entries (every row of a segment named once) when a
    // segment is longer than the window, its rows fit into LDS and the padding of the last segment of
    // a walk does not cost more references than it saves; else one lane group per entry.
    const int64_t E = kTrainThreads / shape.G;
    const int64_t segs_per_walk = (walk_len + E - 1) / E;
    const int64_t R_seg = E + (E + window - 1) + E * window * K;
    const bool by_segments = E >= window + 2 && seg_lds_bytes(shape, window) <= 48 * 1024 &&
                             segs_per_walk * R_seg <= walk_len * R_entry;
    const int64_t R = by_segments ? R_seg : R_entry;
    const int64_t groups_per_walk = by_segments ? segs_per_walk : walk_len;   // reference groups (of R) per walk

    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const Workspace& w = t->ws;
    const int64_t per_walk = static_cast<int64_t>(walk_len) * window;   // sample indices (and neg_out rows) per walk

    auto prep_args = [&](int64_t i) {
        PrepArgs pa{};
        if (i >= n_batches) return pa;   // refs = 0: nothing to prepare
        const int64_t first = i * walks_per_batch;
        const int64_t count = (n_walks - first < walks_per_batch) ? n_walks - first : walks_per_batch;
        const PrepSlot& ps = w.prep[i & 1];
        pa.walks = walks_dev + first * walk_len; pa.walk_len = walk_len; pa.window = window;
        pa.refs = static_cast<uint32_t>(count * groups_per_walk * R); pa.R = static_cast<uint32_t>(R); pa.K = K;
        pa.xrefs = by_segments ? static_cast<uint32_t>(E) : 1u;
        pa.seg_entries = by_segments ? static_cast<uint32_t>(E) : 0u;
        pa.segs_per_walk = static_cast<uint32_t>(segs_per_walk);
        pa.sample_base = sample_base + static_cast<uint64_t>(first * per_walk);
        pa.k0 = static_cast<uint32_t>(t->seed); pa.k1 = static_cast<uint32_t>(t->seed >> 32);
        pa.alias = al ? al->table : nullptr; pa.alias_n = al ? static_cast<uint64_t>(al->n) : 1; pa.alias_base = al ? al->base : 0;
        uint32_t positions = kSweepPerBlock;     // hash positions this batch uses
        while (positions < kHashFactor * pa.refs) positions <<= 1;
        pa.slots = ps.slots; pa.mask = positions - 1; pa.shared = ps.shared; pa.refshared = ps.refshared; pa.ids = ps.ids; pa.posbuf = ps.posbuf;
        pa.neg_out = neg_out_dev ? neg_out_dev + first * per_walk * K : nullptr;
        return pa;
    };

    return run_batches(t, n_batches, R, window, K, lr_host, st, prep_args, [&](const TrainArgs& ta, const PrepArgs& next) {
        return by_segments ? launch_train_seg(shape, ta, next, static_cast<unsigned>(ta.B), st) : launch_train_walk(shape, ta, next, st);
    });
}

ne_status ne_train_batch(ne_tables* t, const ne_alias* al, const int32_t* pairs_dev, int64_t B, int32_t K,
                         float lr, uint64_t sample_base, int32_t* neg_out_dev, void* hip_stream)
{
    if (B == 0) {
        Shape shape;
        return check_batch_args(t, al, pairs_dev, B, K, &shape);
    }
    return ne_train_block(t, al, pairs_dev, B, B, K, &lr, sample_base, neg_out_dev, hip_stream);
}

ne_status ne_train_block_async(ne_tables* t, const ne_alias* al, const int32_t* pairs_dev, int64_t n_pairs, int64_t B,
                               int32_t K, const float* lr_host, uint64_t sample_base, int32_t* neg_out_dev,
                               void* hip_stream)
{
    const ne_run run{al, pairs_dev, n_pairs, sample_base, neg_out_dev};
    return train_runs_impl(t, &run, 1, B, K, lr_host, nullptr, hip_stream, true);
}

ne_status ne_train_batch_async(ne_tables* t, const ne_alias* al, const int32_t* pairs_dev, int64_t B, int32_t K,
                               float lr, uint64_t sample_base, int32_t* neg_out_dev, void* hip_stream)
{
    if (B == 0) {
        Shape shape;
        return check_batch_args(t, al, pairs_dev, B, K, &shape);
    }
    return ne_train_block_async(t, al, pairs_dev, B, B, K, &lr, sample_base, neg_out_dev, hip_stream);
}

ne_status ne_eval_loss(const ne_tables* t, const ne_alias* al, const int32_t* pairs_dev, int64_t B, int32_t K,
                       uint64_t sample_base, double* loss_sum_dev, int32_t* neg_out_dev, void* hip_stream)
{
    Shape shape;
    ne_status rc = check_batch_args(t, al, pairs_dev, B, K, &shape);
    if (rc != NE_OK) return rc;
    if (!loss_sum_dev || !aligned(loss_sum_dev, 8)) return fail(NE_ERR_ARG, "loss_sum_dev is NULL or misaligned");
    if (B == 0) return NE_OK;
    LossArgs la{};
    la.X = reinterpret_cast<const float4*>(t->vertex);
    la.C = reinterpret_cast<const float4*>(t->context);
    la.pairs = reinterpret_cast<const int2*>(pairs_dev);
    la.B = B; la.K = K; la.d4 = t->dim / 4; la.sample_base = sample_base;
    la.k0 = static_cast<uint32_t>(t->seed); la.k1 = static_cast<uint32_t>(t->seed >> 32);
    la.alias = al ? al->table : nullptr; la.alias_n = al ? static_cast<uint64_t>(al->n) : 1; la.alias_base = al ? al->base : 0;
    la.neg_out = neg_out_dev; la.loss = loss_sum_dev;
    hipError_t e = launch_loss(shape, la, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail(NE_ERR_HIP, std::string("loss launch: ") + hipGetErrorString(e));
    return NE_OK;
}

ne_status ne_set_vertex_window(ne_tables* t, float* vertex_window_dev, int64_t first_row, int64_t num_rows)
{
    if (!t) return fail(NE_ERR_ARG, "tables handle is NULL");
    if (!vertex_window_dev || !aligned(vertex_window_dev, 16)) return fail(NE_ERR_ARG, "vertex_window_dev is NULL or not 16-byte aligned");
    if (first_row < 0 || num_rows <= 0 || first_row + num_rows > t->num_nodes)
        return fail(NE_ERR_ARG, "window [first_row, first_row + num_rows) is not inside [0, num_nodes)");
    // the kernels index vertex rows by absolute id: point them at where row 0 would be
    t->vertex = vertex_window_dev - first_row * static_cast<int64_t>(t->dim);
    return NE_OK;
}

ne_status ne_score_pairs(const ne_tables* t, const int32_t* pairs_dev, int64_t n, int32_t second_from_context,
                         float* scores_dev, void* hip_stream)
{
    if (!t) return fail(NE_ERR_ARG, "tables handle is NULL");
    if (n < 0 || n > (static_cast<int64_t>(1) << 40)) return fail(NE_ERR_ARG, "n out of range");
    if (n == 0) return NE_OK;
    if (!pairs_dev || !aligned(pairs_dev, 8)) return fail(NE_ERR_ARG, "pairs_dev is NULL or not 8-byte aligned");
    if (!scores_dev || !aligned(scores_dev, 4)) return fail(NE_ERR_ARG, "scores_dev is NULL or misaligned");
    const int64_t want = (n + 15) / 16;
    const unsigned grid = static_cast<unsigned>(want < 65536 ? want : 65536);
    hipLaunchKernelGGL(score_pairs_kernel, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                       reinterpret_cast<const float4*>(t->vertex),
                       reinterpret_cast<const float4*>(second_from_context ? t->context : t->vertex),
                       reinterpret_cast<const int2*>(pairs_dev), n, t->dim / 4, scores_dev);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(NE_ERR_HIP, std::string("score launch: ") + hipGetErrorString(e));
    return NE_OK;
}

ne_status ne_set_tuning(ne_tables* t, int32_t list_cap, int32_t sweep_per_thread)
{
    if (!t) return fail(NE_ERR_ARG, "tables handle is NULL");
    if (list_cap < -1 || list_cap > static_cast<int32_t>(kListCap)) return fail(NE_ERR_ARG, "list_cap must be -1 (automatic) or in [0, 8]");
    if (sweep_per_thread != 0 && sweep_per_thread != 2 && sweep_per_thread != 4 && sweep_per_thread != 8)
        return fail(NE_ERR_ARG, "sweep_per_thread must be 0 (automatic), 2, 4 or 8");
    t->tune_list_cap = list_cap;
    t->tune_sweep = sweep_per_thread;
    return NE_OK;
}

uint32_t ne_hash_position(uint32_t key, uint32_t positions)
{
    if (positions < 2 || positions > 0x80000000u || (positions & (positions - 1)) != 0) return 0xFFFFFFFFu;
    return hash_position(key, positions - 1);
}

ne_status ne_validate_pairs(const ne_tables* t, const int32_t* pairs_dev, int64_t B,
                            unsigned long long* bad_count_dev, void* hip_stream)
{
    if (!t || !bad_count_dev) return fail(NE_ERR_ARG, "NULL argument");
    if (B < 0 || B > (static_cast<int64_t>(1) << 40)) return fail(NE_ERR_ARG, "B out of range");
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
