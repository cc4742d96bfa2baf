/*
 * CPU oracle for skip-gram-with-negative-sampling (SGNS) node-embedding training.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the GPU
 * library is checked against.  It shares no code, header, table or constant
 * generator with the HIP path and must never be called from the product path.
 *
 * What it follows
 * ---------------
 * The paper (Sec. II-A "Training Process" and Algorithm 1, embedding-training
 * loop) gives the structure: pick a batch of (v,u) edge samples, train
 * (vertex[v], context[u]) with label 1, and for every negative u' train
 * (vertex[v], context[u']) with label 0, by SGD on a similarity score.  Table I
 * fixes the storage: 4-byte node ids, 8-byte (src,dst) samples, fp32 tables.
 * The paper does not state the score, the loss, the negative distribution or
 * the random-number generator; those are the standard SGNS choices:
 *   score      s = <vertex[v], context[u]>
 *   objective  J = log sigma(s_pos) + sum_k log sigma(-s_neg_k)
 *   negatives  P(i) ~ degree_i^0.75 through a Walker/Vose alias table
 *   randomness Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11), counter based
 * Update semantics are minibatch-synchronous: every gradient of a batch is
 * evaluated at the tables as they were before the batch, duplicates are summed,
 * and the sums are applied once.
 *
 * Arithmetic is fp64 everywhere; tables are stored as fp32.
 * No blocking, no reordering: loops are in the order of the maths.  No threads either,
 * but for oracle_train_batch_threads, the same step shared out over host threads
 * so that the oracle can be timed on all cores of a machine.
 *
 * Pins (tests/, -m "not gpu"): finite differences and torch-CPU autograd for the
 * update, closed forms for the loss and for the first batch from a zero context
 * table, exact integer identity + 10^7-draw frequencies for the alias table,
 * rocRAND's host-callable Philox engine and big-integer arithmetic for Philox,
 * hand values and the loss function's positive term for the pair score,
 * a worked example, the sample count of full walks and a brute-force set for the walk samples;
 * oracle_train_batch_threads against the pinned oracle_train_batch.
 * Parity unpinned: none of the functions below.
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------- */
/* Philox4x32-10 (Salmon et al., SC'11): 10 rounds of                         */
/*   (hi0,lo0) = M0*c0, (hi1,lo1) = M1*c2                                     */
/*   c <- (hi1^c1^k0, lo1, hi0^c3^k1, lo0);  k <- k + (W0, W1)                */
/* ------------------------------------------------------------------------- */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = M0 * (uint64_t)c0;
        uint64_t p1 = M1 * (uint64_t)c2;
        uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        uint32_t n0 = hi1 ^ c1 ^ k0;
        uint32_t n1 = lo1;
        uint32_t n2 = hi0 ^ c3 ^ k1;
        uint32_t n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += W0; k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Random-stream ids (4th counter word). */
enum { STREAM_NEGATIVE = 0, STREAM_INIT = 1, STREAM_SHARED_NEGATIVE = 2 };

/* ------------------------------------------------------------------------- */
/* Table initialisation: vertex ~ U(-0.5/d, 0.5/d), context = 0.              */
/* Element (row, col) uses Philox(key = seed, counter = (row_lo, row_hi,      */
/* col/4, STREAM_INIT)), output word col%4:                                   */
/*   u = ((r >> 9) + 0.5) * 2^-23 - 0.5     (open interval, exact in fp32)    */
/*   value = fp32(u / d)                                                       */
/* ------------------------------------------------------------------------- */
void oracle_init_tables(int64_t V, int32_t d, uint64_t seed, float* X, float* C)
{
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    for (int64_t row = 0; row < V; ++row) {
        for (int32_t col = 0; col < d; ++col) {
            uint32_t ctr[4] = { (uint32_t)row, (uint32_t)((uint64_t)row >> 32),
                                (uint32_t)(col / 4), STREAM_INIT };
            uint32_t r[4];
            oracle_philox4x32_10(ctr, key, r);
            double u = ((double)(r[col % 4] >> 9) + 0.5) * (1.0 / 8388608.0) - 0.5;
            X[row * d + col] = (float)(u / (double)d);
            C[row * d + col] = 0.0f;
        }
    }
}

/* ------------------------------------------------------------------------- */
/* Alias table for P(i) ~ degree_i^0.75, i in [0, n).                          */
/*   w_i = sqrt(deg) * sqrt(sqrt(deg))   (fp64, correctly rounded pieces)     */
/*   W   = sum of w_i, left to right                                           */
/*   p_i = (w_i * n) / W                                                       */
/* Vose's construction with two LIFO stacks filled in ascending i:            */
/*   pop s from small, l from large; thr[s] = p_s, alias[s] = l;               */
/*   p_l = (p_l + p_s) - 1; push l to small if p_l < 1 else to large.          */
/* Whatever is left gets thr = 1, alias = itself.                              */
/* Quantisation: thr_q = min(floor(thr * 2^32), 2^32 - 1).                     */
/* prob_out (optional) receives w_i / W.  Returns 0, or -1 if W == 0 / n <= 0. */
/* ------------------------------------------------------------------------- */
int oracle_build_alias(const uint32_t* degree, int64_t n, uint32_t* thr_q, uint32_t* alias,
                       double* prob_out)
{
    if (n <= 0) return -1;
    double* p = (double*)malloc((size_t)n * sizeof(double));
    double* thr = (double*)malloc((size_t)n * sizeof(double));
    int64_t* small = (int64_t*)malloc((size_t)n * sizeof(int64_t));
    int64_t* large = (int64_t*)malloc((size_t)n * sizeof(int64_t));
    if (!p || !thr || !small || !large) { free(p); free(thr); free(small); free(large); return -2; }

    double W = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double deg = (double)degree[i];
        p[i] = sqrt(deg) * sqrt(sqrt(deg));
        W += p[i];
    }
    if (!(W > 0.0)) { free(p); free(thr); free(small); free(large); return -1; }
    for (int64_t i = 0; i < n; ++i) {
        if (prob_out) prob_out[i] = p[i] / W;
        p[i] = (p[i] * (double)n) / W;
    }
    int64_t ns = 0, nl = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (p[i] < 1.0) small[ns++] = i; else large[nl++] = i;
    }
    while (ns > 0 && nl > 0) {
        int64_t s = small[--ns];
        int64_t l = large[--nl];
        thr[s] = p[s];
        alias[s] = (uint32_t)l;
        p[l] = (p[l] + p[s]) - 1.0;
        if (p[l] < 1.0) small[ns++] = l; else large[nl++] = l;
    }
    while (nl > 0) { int64_t l = large[--nl]; thr[l] = 1.0; alias[l] = (uint32_t)l; }
    while (ns > 0) { int64_t s = small[--ns]; thr[s] = 1.0; alias[s] = (uint32_t)s; }

    for (int64_t i = 0; i < n; ++i) {
        double q = floor(thr[i] * 4294967296.0);
        if (q > 4294967295.0) q = 4294967295.0;
        if (q < 0.0) q = 0.0;
        thr_q[i] = (uint32_t)q;
    }
    free(p); free(thr); free(small); free(large);
    return 0;
}

/* One alias draw from the four Philox words:                                  */
/*   slot = floor(((r0 << 32) | r1) * n / 2^64);  keep slot iff r2 < thr_q.    */
static int64_t alias_draw(const uint32_t r[4], const uint32_t* thr_q, const uint32_t* alias,
                          int64_t n)
{
    unsigned __int128 u = ((unsigned __int128)r[0] << 32) | (unsigned __int128)r[1];
    int64_t slot = (int64_t)((u * (unsigned __int128)(uint64_t)n) >> 64);
    return (r[2] < thr_q[slot]) ? slot : (int64_t)alias[slot];
}

/* Negative ids for pairs sample_base .. sample_base+B-1 (Algorithm 1, the     */
/* NegativeSample step): neg[b][k] = base + draw(Philox(seed;                  */
/* counter = (idx_lo, idx_hi, k, STREAM_NEGATIVE))), idx = sample_base + b.    */
void oracle_sample_negatives(uint64_t seed, uint64_t sample_base, int64_t B, int32_t K,
                             const uint32_t* thr_q, const uint32_t* alias, int64_t n,
                             int32_t base, int32_t* neg_out)
{
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    for (int64_t b = 0; b < B; ++b) {
        uint64_t idx = sample_base + (uint64_t)b;
        for (int32_t k = 0; k < K; ++k) {
            uint32_t ctr[4] = { (uint32_t)idx, (uint32_t)(idx >> 32), (uint32_t)k, STREAM_NEGATIVE };
            uint32_t r[4];
            oracle_philox4x32_10(ctr, key, r);
            neg_out[b * K + k] = base + (int32_t)alias_draw(r, thr_q, alias, n);
        }
    }
}

/* Shared negatives of one batch: ids[j] = base + draw(Philox(seed;            */
/* counter = (batch_lo, batch_hi, j, STREAM_SHARED_NEGATIVE))).                */
void oracle_sample_shared_negatives(uint64_t seed, uint64_t batch_index, int32_t N,
                                    const uint32_t* thr_q, const uint32_t* alias, int64_t n,
                                    int32_t base, int32_t* neg_out)
{
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    for (int32_t j = 0; j < N; ++j) {
        uint32_t ctr[4] = { (uint32_t)batch_index, (uint32_t)(batch_index >> 32), (uint32_t)j,
                            STREAM_SHARED_NEGATIVE };
        uint32_t r[4];
        oracle_philox4x32_10(ctr, key, r);
        neg_out[j] = base + (int32_t)alias_draw(r, thr_q, alias, n);
    }
}

static double sigmoid(double z) { return 1.0 / (1.0 + exp(-z)); }
static double softplus(double z) { return (z > 0.0 ? z : 0.0) + log1p(exp(-fabs(z))); }

/* Sparse fp64 accumulator over table rows: slot_of[row] is -1 or an index     */
/* into acc (rows appended in first-touch order).                              */
typedef struct { int64_t* slot_of; int64_t* rows; double* acc; int64_t count, cap; int32_t d; } delta_map;

static int dm_init(delta_map* m, int64_t V, int64_t cap, int32_t d)
{
    m->slot_of = (int64_t*)malloc((size_t)V * sizeof(int64_t));
    m->rows = (int64_t*)malloc((size_t)(cap > 0 ? cap : 1) * sizeof(int64_t));
    m->acc = (double*)malloc((size_t)(cap > 0 ? cap : 1) * (size_t)d * sizeof(double));   /* a row is zeroed when first touched */
    m->count = 0; m->cap = cap; m->d = d;
    if (!m->slot_of || !m->rows || !m->acc) return -1;
    for (int64_t i = 0; i < V; ++i) m->slot_of[i] = -1;
    return 0;
}
static double* dm_row(delta_map* m, int64_t row)
{
    if (m->slot_of[row] < 0) {
        m->slot_of[row] = m->count; m->rows[m->count] = row;
        memset(m->acc + m->count * (int64_t)m->d, 0, (size_t)m->d * sizeof(double));
        m->count++;
    }
    return m->acc + m->slot_of[row] * (int64_t)m->d;
}
static void dm_free(delta_map* m) { free(m->slot_of); free(m->rows); free(m->acc); }

/* ------------------------------------------------------------------------- */
/* One minibatch-synchronous SGNS step (Algorithm 1, embedding-training loop;  */
/* Sec. II-A "Training Process").  pairs = int32[B][2] = (src, ctx);           */
/* neg = int32[B][K].  With x = X[src], c_0 = C[ctx], c_k = C[neg_k], all as   */
/* they are before the batch:                                                  */
/*   s_j = <x, c_j>;  g_0 = 1 - sigma(s_0) (label 1);  g_k = -sigma(s_k)       */
/*   DX[src] += lr * sum_j g_j c_j;   DC[id_j] += lr * g_j x                    */
/* and after all pairs  X += DX, C += DC  (rounded to fp32 once per element).  */
/* Rows no pair names are not written.  Returns 0, -1 on a bad id, -2 no mem.  */
/* ------------------------------------------------------------------------- */
int oracle_train_batch(float* X, float* C, int64_t V, int32_t d, const int32_t* pairs, int64_t B,
                       int32_t K, float lr_f, const int32_t* neg)
{
    const double lr = (double)lr_f;
    for (int64_t b = 0; b < B; ++b) {
        if (pairs[2 * b] < 0 || pairs[2 * b] >= V || pairs[2 * b + 1] < 0 || pairs[2 * b + 1] >= V) return -1;
        for (int32_t k = 0; k < K; ++k)
            if (neg[b * K + k] < 0 || neg[b * K + k] >= V) return -1;
    }
    delta_map DX, DC;
    if (dm_init(&DX, V, B, d) || dm_init(&DC, V, B * (int64_t)(K + 1), d)) { dm_free(&DX); dm_free(&DC); return -2; }

    for (int64_t b = 0; b < B; ++b) {
        const int64_t src = pairs[2 * b];
        const float* x = X + src * (int64_t)d;
        double* dx = dm_row(&DX, src);
        for (int32_t j = 0; j <= K; ++j) {
            const int64_t id = (j == 0) ? pairs[2 * b + 1] : neg[b * K + (j - 1)];
            const float* c = C + id * (int64_t)d;
            double s = 0.0;
            for (int32_t i = 0; i < d; ++i) s += (double)x[i] * (double)c[i];
            const double g = (j == 0) ? 1.0 - sigmoid(s) : -sigmoid(s);
            double* dc = dm_row(&DC, id);
            for (int32_t i = 0; i < d; ++i) {
                dx[i] += lr * g * (double)c[i];
                dc[i] += lr * g * (double)x[i];
            }
        }
    }
    for (int64_t t = 0; t < DX.count; ++t) {
        float* row = X + DX.rows[t] * (int64_t)d;
        for (int32_t i = 0; i < d; ++i) row[i] = (float)((double)row[i] + DX.acc[t * (int64_t)d + i]);
    }
    for (int64_t t = 0; t < DC.count; ++t) {
        float* row = C + DC.rows[t] * (int64_t)d;
        for (int32_t i = 0; i < d; ++i) row[i] = (float)((double)row[i] + DC.acc[t * (int64_t)d + i]);
    }
    dm_free(&DX); dm_free(&DC);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* The same step with the pairs spread over host threads, for timing the       */
/* oracle on all cores of a machine next to the one-thread figure.  Thread t   */
/* takes the t-th contiguous share of the pairs and accumulates, exactly as    */
/* above, into delta maps of its own; then every thread adds up, in the order  */
/* of the threads, all threads' sums for the rows it owns (row % threads) and  */
/* applies them.  Only the order of the fp64 sums differs from                 */
/* oracle_train_batch (pinned to it in tests/).                                */
/* Returns 0, -1 on a bad id, -2 no memory, -3 thread creation failed.         */
/* ------------------------------------------------------------------------- */
typedef struct share_job {
    float* X; float* C; int32_t d; const int32_t* pairs; int32_t K; double lr; const int32_t* neg;
    int64_t b0, b1;                 /* this thread's share of the pairs                          */
    delta_map DX, DC;               /* its own sums over that share                              */
    delta_map GX, GC;               /* totals of the rows it owns (row % T == its index)         */
    struct share_job* all; int64_t T, self;
} share_job;

/* Phase 1: the loop of oracle_train_batch over this thread's share of the pairs. */
static void* share_accumulate(void* arg)
{
    share_job* jb = (share_job*)arg;
    const int32_t d = jb->d, K = jb->K;
    for (int64_t b = jb->b0; b < jb->b1; ++b) {
        const int64_t src = jb->pairs[2 * b];
        const float* x = jb->X + src * (int64_t)d;
        double* dx = dm_row(&jb->DX, src);
        for (int32_t j = 0; j <= K; ++j) {
            const int64_t id = (j == 0) ? jb->pairs[2 * b + 1] : jb->neg[b * K + (j - 1)];
            const float* c = jb->C + id * (int64_t)d;
            double s = 0.0;
            for (int32_t i = 0; i < d; ++i) s += (double)x[i] * (double)c[i];
            const double g = (j == 0) ? 1.0 - sigmoid(s) : -sigmoid(s);
            double* dc = dm_row(&jb->DC, id);
            for (int32_t i = 0; i < d; ++i) {
                dx[i] += jb->lr * g * (double)c[i];
                dc[i] += jb->lr * g * (double)x[i];
            }
        }
    }
    return NULL;
}

/* Phase 2: this thread adds up, in the order of the threads, every thread's sums for the rows it   */
/* owns, and applies the totals to the tables (one rounding to fp32 per element).                  */
static void* share_merge(void* arg)
{
    share_job* me = (share_job*)arg;
    const int32_t d = me->d;
    for (int64_t t = 0; t < me->T; ++t) {
        const share_job* src = &me->all[t];
        for (int64_t r = 0; r < src->DX.count; ++r) {
            if (src->DX.rows[r] % me->T != me->self) continue;
            double* g = dm_row(&me->GX, src->DX.rows[r]);
            for (int32_t i = 0; i < d; ++i) g[i] += src->DX.acc[r * (int64_t)d + i];
        }
        for (int64_t r = 0; r < src->DC.count; ++r) {
            if (src->DC.rows[r] % me->T != me->self) continue;
            double* g = dm_row(&me->GC, src->DC.rows[r]);
            for (int32_t i = 0; i < d; ++i) g[i] += src->DC.acc[r * (int64_t)d + i];
        }
    }
    for (int64_t t = 0; t < me->GX.count; ++t) {
        float* row = me->X + me->GX.rows[t] * (int64_t)d;
        for (int32_t i = 0; i < d; ++i) row[i] = (float)((double)row[i] + me->GX.acc[t * (int64_t)d + i]);
    }
    for (int64_t t = 0; t < me->GC.count; ++t) {
        float* row = me->C + me->GC.rows[t] * (int64_t)d;
        for (int32_t i = 0; i < d; ++i) row[i] = (float)((double)row[i] + me->GC.acc[t * (int64_t)d + i]);
    }
    return NULL;
}

static int run_on_threads(share_job* jobs, pthread_t* tid, int64_t T, void* (*fn)(void*))
{
    int64_t started = 0;
    int rc = 0;
    for (int64_t t = 0; t < T; ++t, ++started)
        if (pthread_create(&tid[t], NULL, fn, &jobs[t]) != 0) { rc = -3; break; }
    for (int64_t t = 0; t < started; ++t) pthread_join(tid[t], NULL);
    return rc;
}

/* (Not reentrant: one call at a time per process.)                                                  */
/* Memory of thread t's four delta maps, kept from one call to the next (fresh pages cost more than   */
/* the arithmetic when every call maps and unmaps a few hundred MB per thread).  slot_of is all -1    */
/* between calls: a call resets the entries it has set.                                               */
enum { MAX_SHARE_THREADS = 256 };
static struct { char* base; size_t bytes; int64_t V, d, cap[4]; } share_pool[MAX_SHARE_THREADS];   /* cap: the layout it holds */

static char* pool_take(char** cur, size_t bytes) { char* p = *cur; *cur += (bytes + 63) & ~(size_t)63; return p; }
static void pool_map(delta_map* m, char** cur, int64_t V, int64_t cap, int32_t d)
{
    m->slot_of = (int64_t*)pool_take(cur, (size_t)V * sizeof(int64_t));
    m->rows = (int64_t*)pool_take(cur, (size_t)(cap > 0 ? cap : 1) * sizeof(int64_t));
    m->acc = (double*)pool_take(cur, (size_t)(cap > 0 ? cap : 1) * (size_t)d * sizeof(double));
    m->count = 0; m->cap = cap; m->d = d;
}
static void pool_reset(delta_map* m) { for (int64_t r = 0; r < m->count; ++r) m->slot_of[m->rows[r]] = -1; }

int oracle_train_batch_threads(float* X, float* C, int64_t V, int32_t d, const int32_t* pairs, int64_t B,
                               int32_t K, float lr_f, const int32_t* neg, int32_t threads)
{
    for (int64_t b = 0; b < B; ++b) {
        if (pairs[2 * b] < 0 || pairs[2 * b] >= V || pairs[2 * b + 1] < 0 || pairs[2 * b + 1] >= V) return -1;
        for (int32_t k = 0; k < K; ++k)
            if (neg[b * K + k] < 0 || neg[b * K + k] >= V) return -1;
    }
    int64_t T = threads < 1 ? 1 : (threads > MAX_SHARE_THREADS ? MAX_SHARE_THREADS : threads);
    if (T > B) T = B > 0 ? B : 1;
    share_job* jobs = (share_job*)calloc((size_t)T, sizeof(share_job));
    pthread_t* tid = (pthread_t*)calloc((size_t)T, sizeof(pthread_t));
    int rc = 0;
    if (!jobs || !tid) { free(jobs); free(tid); return -2; }
    for (int64_t t = 0; t < T && rc == 0; ++t) {
        share_job* jb = &jobs[t];
        jb->X = X; jb->C = C; jb->d = d; jb->pairs = pairs; jb->K = K; jb->lr = (double)lr_f; jb->neg = neg;
        jb->b0 = B * t / T; jb->b1 = B * (t + 1) / T;
        jb->all = jobs; jb->T = T; jb->self = t;
        const int64_t n = jb->b1 - jb->b0;
        /* a thread owns at most min(rows named, its share of V) rows */
        const int64_t own = (V + T - 1) / T;
        const int64_t cap[4] = { n, n * (int64_t)(K + 1), B < own ? B : own,
                                 B * (int64_t)(K + 1) < own ? B * (int64_t)(K + 1) : own };
        size_t need = 0;
        for (int i = 0; i < 4; ++i)
            need += (((size_t)V * 8 + 63) & ~(size_t)63) + (((size_t)(cap[i] > 0 ? cap[i] : 1) * 8 + 63) & ~(size_t)63) +
                    (((size_t)(cap[i] > 0 ? cap[i] : 1) * (size_t)d * 8 + 63) & ~(size_t)63);
        /* same layout as the last call: the slot_of arrays are where they were, all -1 */
        int fresh = share_pool[t].V != V || share_pool[t].d != d;
        for (int i = 0; i < 4; ++i) fresh = fresh || share_pool[t].cap[i] != cap[i];
        if (share_pool[t].bytes < need) {
            free(share_pool[t].base);
            share_pool[t].base = (char*)malloc(need);
            share_pool[t].bytes = share_pool[t].base ? need : 0;
            fresh = 1;
            if (!share_pool[t].base) { share_pool[t].V = 0; rc = -2; break; }
        }
        share_pool[t].V = V; share_pool[t].d = d;
        for (int i = 0; i < 4; ++i) share_pool[t].cap[i] = cap[i];
        char* cur = share_pool[t].base;
        delta_map* maps[4] = { &jb->DX, &jb->DC, &jb->GX, &jb->GC };
        for (int i = 0; i < 4; ++i) {
            pool_map(maps[i], &cur, V, cap[i], d);
            if (fresh) for (int64_t r = 0; r < V; ++r) maps[i]->slot_of[r] = -1;
        }
    }
    if (rc == 0) rc = run_on_threads(jobs, tid, T, share_accumulate);
    if (rc == 0) rc = run_on_threads(jobs, tid, T, share_merge);
    for (int64_t t = 0; t < T; ++t)
        if (share_pool[t].base && jobs[t].DX.slot_of) {
            pool_reset(&jobs[t].DX); pool_reset(&jobs[t].DC); pool_reset(&jobs[t].GX); pool_reset(&jobs[t].GC);
        }
    free(jobs); free(tid);
    return rc;
}

/* Loss of a batch at the current tables, summed over pairs (not averaged):    */
/*   sum_b [ -log sigma(s_b0) - sum_k log sigma(-s_bk) ]                        */
/* written with softplus(z) = log(1 + e^z):  softplus(-s_0) + sum softplus(s_k) */
double oracle_eval_loss(const float* X, const float* C, int64_t V, int32_t d, const int32_t* pairs,
                        int64_t B, int32_t K, const int32_t* neg)
{
    (void)V;
    double total = 0.0;
    for (int64_t b = 0; b < B; ++b) {
        const float* x = X + (int64_t)pairs[2 * b] * d;
        for (int32_t j = 0; j <= K; ++j) {
            const int64_t id = (j == 0) ? pairs[2 * b + 1] : neg[b * K + (j - 1)];
            const float* c = C + id * (int64_t)d;
            double s = 0.0;
            for (int32_t i = 0; i < d; ++i) s += (double)x[i] * (double)c[i];
            total += (j == 0) ? softplus(-s) : softplus(s);
        }
    }
    return total;
}

/* ------------------------------------------------------------------------- */
/* Shared-negative mode (the level-3-BLAS formulation the paper cites as       */
/* related work, Sec. VI-B: the negatives are shared by a whole mini-batch so  */
/* that scoring becomes a dense product).  All B pairs of the batch are scored */
/* against the same N negative rows; every negative term carries the weight    */
/* neg_scale:                                                                  */
/*   J = sum_b [ log sigma(x_b . c_ctx_b) + neg_scale sum_n log sigma(-x_b . c_n) ] */
/* Positive part exactly as in oracle_train_batch (full precision).            */
/* Negative part, with q() = round-to-nearest-even to bfloat16 when            */
/* bf16_inputs != 0 (identity otherwise):                                      */
/*   S_bn = <q(x_b), q(c_n)>;  G_bn = q(fp32(-neg_scale sigma(S_bn)))           */
/*   DX[src_b] += lr sum_n G_bn q(c_n);   DC[neg_n] += lr sum_b G_bn q(x_b)      */
/* All deltas from the pre-batch tables, summed, applied once.  *loss_out (if  */
/* not NULL) receives sum_b [softplus(-s_b0) + neg_scale sum_n softplus(S_bn)]. */
/* ------------------------------------------------------------------------- */
static float bf16_rne(float x)
{
    uint32_t u;
    memcpy(&u, &x, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    u &= 0xFFFF0000u;
    float r;
    memcpy(&r, &u, 4);
    return r;
}

int oracle_train_batch_shared(float* X, float* C, int64_t V, int32_t d, const int32_t* pairs, int64_t B,
                              const int32_t* negs, int32_t N, float lr_f, float neg_scale_f,
                              int32_t bf16_inputs, double* loss_out)
{
    const double lr = (double)lr_f, neg_scale = (double)neg_scale_f;
    for (int64_t b = 0; b < B; ++b)
        if (pairs[2 * b] < 0 || pairs[2 * b] >= V || pairs[2 * b + 1] < 0 || pairs[2 * b + 1] >= V) return -1;
    for (int32_t n = 0; n < N; ++n)
        if (negs[n] < 0 || negs[n] >= V) return -1;
    delta_map DX, DC;
    if (dm_init(&DX, V, B, d) || dm_init(&DC, V, B + N, d)) { dm_free(&DX); dm_free(&DC); return -2; }
    double* xq = (double*)malloc((size_t)d * sizeof(double));
    double* cq = (double*)malloc((size_t)d * sizeof(double));
    if (!xq || !cq) { free(xq); free(cq); dm_free(&DX); dm_free(&DC); return -2; }
    double loss = 0.0;

    for (int64_t b = 0; b < B; ++b) {
        const int64_t src = pairs[2 * b], ctx = pairs[2 * b + 1];
        const float* x = X + src * (int64_t)d;
        const float* c0 = C + ctx * (int64_t)d;
        double* dx = dm_row(&DX, src);
        /* positive pair, label 1 */
        double s0 = 0.0;
        for (int32_t i = 0; i < d; ++i) s0 += (double)x[i] * (double)c0[i];
        const double g0 = 1.0 - sigmoid(s0);
        loss += softplus(-s0);
        double* dc0 = dm_row(&DC, ctx);
        for (int32_t i = 0; i < d; ++i) {
            dx[i] += lr * g0 * (double)c0[i];
            dc0[i] += lr * g0 * (double)x[i];
        }
        /* shared negatives, label 0, weight neg_scale */
        for (int32_t i = 0; i < d; ++i) xq[i] = bf16_inputs ? (double)bf16_rne(x[i]) : (double)x[i];
        for (int32_t n = 0; n < N; ++n) {
            const float* c = C + (int64_t)negs[n] * d;
            double S = 0.0;
            for (int32_t i = 0; i < d; ++i) {
                cq[i] = bf16_inputs ? (double)bf16_rne(c[i]) : (double)c[i];
                S += xq[i] * cq[i];
            }
            loss += neg_scale * softplus(S);
            double G = -neg_scale * sigmoid(S);
            if (bf16_inputs) G = (double)bf16_rne((float)G);
            double* dc = dm_row(&DC, negs[n]);
            for (int32_t i = 0; i < d; ++i) {
                dx[i] += lr * G * cq[i];
                dc[i] += lr * G * xq[i];
            }
        }
    }
    for (int64_t t = 0; t < DX.count; ++t) {
        float* row = X + DX.rows[t] * (int64_t)d;
        for (int32_t i = 0; i < d; ++i) row[i] = (float)((double)row[i] + DX.acc[t * (int64_t)d + i]);
    }
    for (int64_t t = 0; t < DC.count; ++t) {
        float* row = C + DC.rows[t] * (int64_t)d;
        for (int32_t i = 0; i < d; ++i) row[i] = (float)((double)row[i] + DC.acc[t * (int64_t)d + i]);
    }
    if (loss_out) *loss_out = loss;
    free(xq); free(cq);
    dm_free(&DX); dm_free(&DC);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Per-sample ("asynchronous") training: the loop of Algorithm 1 taken         */
/* literally, one edge sample after the other, each seeing the tables as the   */
/* samples before it left them.  Within one sample the K+1 Train calls use the */
/* source row as it was when the sample started and the source row is updated  */
/* once with the summed gradient (the word2vec convention); context rows are   */
/* updated after the sample's scores are formed.  This is the reference for    */
/* the GPU's unsynchronised mode, which is compared statistically (loss curve) */
/* and, on batches in which no row is named twice, element by element.         */
/* ------------------------------------------------------------------------- */
int oracle_train_sequential(float* X, float* C, int64_t V, int32_t d, const int32_t* pairs, int64_t B,
                            int32_t K, float lr_f, const int32_t* neg)
{
    const double lr = (double)lr_f;
    double* dx = (double*)malloc((size_t)d * sizeof(double));
    double* g = (double*)malloc((size_t)(K + 1) * sizeof(double));
    double* xs = (double*)malloc((size_t)d * sizeof(double));
    if (!dx || !g || !xs) { free(dx); free(g); free(xs); return -2; }
    for (int64_t b = 0; b < B; ++b) {
        const int64_t src = pairs[2 * b];
        if (src < 0 || src >= V) { free(dx); free(g); free(xs); return -1; }
        float* x = X + src * (int64_t)d;
        for (int32_t i = 0; i < d; ++i) { dx[i] = 0.0; xs[i] = (double)x[i]; }
        for (int32_t j = 0; j <= K; ++j) {
            const int64_t id = (j == 0) ? pairs[2 * b + 1] : neg[b * K + (j - 1)];
            if (id < 0 || id >= V) { free(dx); free(g); free(xs); return -1; }
            const float* c = C + id * (int64_t)d;
            double s = 0.0;
            for (int32_t i = 0; i < d; ++i) s += xs[i] * (double)c[i];
            g[j] = (j == 0) ? 1.0 - sigmoid(s) : -sigmoid(s);
            for (int32_t i = 0; i < d; ++i) dx[i] += lr * g[j] * (double)c[i];
        }
        for (int32_t j = 0; j <= K; ++j) {
            const int64_t id = (j == 0) ? pairs[2 * b + 1] : neg[b * K + (j - 1)];
            float* c = C + id * (int64_t)d;
            for (int32_t i = 0; i < d; ++i) c[i] = (float)((double)c[i] + lr * g[j] * xs[i]);
        }
        for (int32_t i = 0; i < d; ++i) x[i] = (float)(xs[i] + dx[i]);
    }
    free(dx); free(g); free(xs);
    return 0;
}

/* Similarity score of arbitrary node pairs (evaluation for link prediction, Sec. V-B): the dot
 * product of the first node's vertex row with the second node's context row (second_from_context)
 * or vertex row, accumulated in fp64 in index order. */
void oracle_score_pairs(const float* X, const float* C, int32_t d, const int32_t* pairs, int64_t n,
                        int32_t second_from_context, double* scores_out)
{
    const float* S = second_from_context ? C : X;
    for (int64_t i = 0; i < n; ++i) {
        const float* a = X + (int64_t)pairs[2 * i] * d;
        const float* b = S + (int64_t)pairs[2 * i + 1] * d;
        double acc = 0.0;
        for (int32_t k = 0; k < d; ++k) acc += (double)a[k] * (double)b[k];
        scores_out[i] = acc;
    }
}

/* Network augmentation (Algorithm 1): the samples of a set of walks.  Entry i of a walk is the source
 * of the samples (walk[i], walk[i+j]) for 1 <= j <= window with i + j < walk_len; the earlier node
 * is the source; a sample exists only if both entries are non-negative.  Samples are listed by walk,
 * then entry, then offset; sample_out receives  (r * walk_len + i) * window + (j - 1)  for each, the
 * index its negatives are drawn for (relative to the call's first sample index).  pairs_out and
 * sample_out need room for n_walks * walk_len * window samples.  Returns the number of samples. */
int64_t oracle_walk_pairs(const int32_t* walks, int64_t n_walks, int32_t walk_len, int32_t window,
                          int32_t* pairs_out, int64_t* sample_out)
{
    int64_t n = 0;
    for (int64_t r = 0; r < n_walks; ++r) {
        const int32_t* w = walks + r * (int64_t)walk_len;
        for (int32_t i = 0; i < walk_len; ++i) {
            for (int32_t j = 1; j <= window; ++j) {
                if (i + j >= walk_len) continue;
                if (w[i] < 0 || w[i + j] < 0) continue;
                pairs_out[2 * n] = w[i];
                pairs_out[2 * n + 1] = w[i + j];
                sample_out[n] = (r * (int64_t)walk_len + i) * (int64_t)window + (j - 1);
                ++n;
            }
        }
    }
    return n;
}
