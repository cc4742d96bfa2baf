/*
 * ne.h - C ABI of the MI355X (gfx950) SGNS node-embedding training library.
 *
 * The library runs the embedding-training loop of the paper's Algorithm 1 (Sec. II-A "Training
 * Process") on one GPU: for a batch of positive (src, ctx) edge samples it draws K negative context
 * nodes per sample, scores vertex[src] against context[ctx] (label 1) and context[neg_k] (label 0)
 * with a dot product and a sigmoid, and applies the SGD update to both embedding tables.  Data
 * formats follow Table I: node ids are 4 bytes, a sample is an 8-byte (src, ctx) pair, and both
 * embedding tables are row-major fp32 [num_nodes][dim].
 *
 * Update semantics are minibatch-synchronous: every gradient of a batch is evaluated at the tables
 * as they were before the batch, contributions to the same row are summed, and the sums are applied
 * once (across GPUs the paper's training is synchronous as well, Sec. III-B; inside a GPU it fixes
 * nothing).
 *
 * Conventions
 *  - "_dev" pointers are device memory owned by the caller; "_host" pointers are host memory.  The
 *    library never allocates or frees device memory: scratch comes in as a workspace argument.
 *    The opaque handles are small host structs.
 *  - hip_stream is a hipStream_t passed as void* (NULL = the default stream).  Unless stated
 *    otherwise a call enqueues its work on that stream and returns without synchronising.
 *  - Every call returns NE_OK or a negative ne_status.  Argument errors are detected on the host
 *    before anything is enqueued.  ne_last_error() describes the last failure on this thread.
 *  - Node ids inside pairs_dev are not range-checked on the training path; ne_validate_pairs does it.
 *  - Random draws are Philox4x32-10 (Salmon et al., SC'11) keyed by the tables' seed and addressed
 *    by (sample index, k), so results do not depend on how samples are split into calls.
 */
#ifndef NE_H
#define NE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ne_tables ne_tables; /* host handle: pointers + shape of the two embedding tables   */
typedef struct ne_alias ne_alias;   /* host handle: a device alias table over ids [base, base+n)   */

typedef enum {
    NE_OK = 0,
    NE_ERR_ARG = -1,   /* bad argument (null pointer, shape, range, too-small buffer)              */
    NE_ERR_STATE = -2, /* handles that do not belong together                                      */
    NE_ERR_HIP = -3,   /* a HIP runtime call or kernel launch failed                               */
    NE_ERR_NOMEM = -4  /* host allocation failed                                                   */
} ne_status;

enum { NE_MAX_DIM = 1024, NE_MAX_NEGATIVES = 62, NE_MAX_BATCH = 1 << 22 };

/* Bytes of device workspace a tables handle needs to train batches of up to max_batch pairs with up
 * to max_negatives negatives each (0 if an argument is invalid). */
size_t ne_workspace_bytes(int32_t dim, int64_t max_batch, int32_t max_negatives);

/*
 * Bind the vertex and context embedding matrices of Sec. II-A ("Embedding Representation") and,
 * if init != 0, initialise them on the stream: vertex ~ U(-0.5/dim, 0.5/dim), context = 0.
 * Element (row, col) of vertex is ((r >> 9) + 0.5) * 2^-23 - 0.5, divided by dim, where r is output
 * word col%4 of Philox(key = seed, counter = (row, 0, col/4, 1)).
 *   vertex_dev, context_dev : device, fp32 [num_nodes][dim] row-major, 16-byte aligned, caller-owned,
 *                             must stay valid while the handle is used.
 *   0 < num_nodes < 2^31;  dim % 4 == 0, 4 <= dim <= NE_MAX_DIM.
 *   seed keys every random draw made through this handle.
 *   workspace_dev : device scratch for ne_train_batch, 256-byte aligned, at least
 *                   ne_workspace_bytes(dim, max_batch, max_negatives) bytes, caller-owned, used only
 *                   through this handle until the handle is destroyed; it is cleared on the stream
 *                   here.  Pass NULL with max_batch = 0 for a handle that is only evaluated.
 *   1 <= max_batch <= NE_MAX_BATCH, 0 <= max_negatives <= NE_MAX_NEGATIVES when training.
 * *out receives a handle to free with ne_destroy_tables.  Errors: NE_ERR_ARG, NE_ERR_NOMEM, NE_ERR_HIP.
 */
ne_status ne_create_tables(ne_tables** out, int64_t num_nodes, int32_t dim, float* vertex_dev,
                           float* context_dev, uint64_t seed, int32_t init, int64_t max_batch,
                           int32_t max_negatives, void* workspace_dev, size_t workspace_bytes,
                           void* hip_stream);

/*
 * Build the negative-sampling table (Algorithm 1, NegativeSample) for the id range [base, base+n):
 * P(base+i) proportional to degree_host[i]^0.75, as a Walker/Vose alias table of n entries
 * {uint32 threshold, uint32 alias} (8 bytes each) written to alias_dev.
 *   degree_host : host, uint32[n], read during the call only.  At least one entry must be non-zero.
 *   alias_dev   : device, 8*n bytes, 8-byte aligned, caller-owned, must outlive the handle's use.
 *   0 < n, 0 <= base, base + n < 2^31.
 * The table is built on the host (fp64, sequential, deterministic) and copied on the stream; the
 * call returns after the copy has completed.  A draw uses the four Philox words r0..r3:
 * slot = floor(((r0<<32)|r1) * n / 2^64); id = base + (r2 < threshold[slot] ? slot : alias[slot]).
 * Errors: NE_ERR_ARG (also when all degrees are zero), NE_ERR_NOMEM, NE_ERR_HIP.
 */
ne_status ne_build_neg_alias(ne_alias** out, const uint32_t* degree_host, int64_t n, int32_t base,
                             void* alias_dev, void* hip_stream);

/*
 * One minibatch-synchronous SGNS step (Algorithm 1, one iteration of the embedding-training loop
 * for every pair of the batch).
 *   pairs_dev   : device, int32[B][2] = (src, ctx), 8-byte aligned; ids must lie in [0, num_nodes).
 *   B           : 0 <= B <= max_batch of the handle.  B == 0 is a no-op.
 *   K           : negatives per pair, 0 <= K <= max_negatives of the handle.  Negative k of pair b is
 *                 the alias draw for Philox(key = seed, counter = (idx_lo, idx_hi, k, 0)),
 *                 idx = sample_base + b.  The alias range must lie inside [0, num_nodes).
 *   lr          : learning rate of this batch (the caller owns the schedule).
 *   neg_out_dev : NULL, or device int32[B][K] that receives the negative ids used.
 * With x = vertex[src], c_0 = context[ctx], c_k = context[neg_k] read before the batch:
 *   s_j = <x, c_j>,  g_0 = 1 - sigmoid(s_0),  g_k = -sigmoid(s_k),
 *   vertex[src] += lr * sum_j g_j c_j,   context[id_j] += lr * g_j x,
 * contributions to the same row summed (in fp32; the order of the sum is not fixed).
 * Accuracy: a row that one reference of the batch names is updated with one rounding per element.  A row
 * that n references name has their n deltas added one after the other in fp32, so its update carries an
 * accumulation error of up to about n * 2^-24 of the summed magnitudes: typically sqrt(n) * 2^-24, close
 * to the bound when many of the contributions are identical (the same source row against the same context
 * row many times).  Up to n of about 1700 that is inside a relative error of 1e-4 per row; a hub row that
 * tens of thousands of samples of one batch name can exceed it (1.7e-4 measured at n = 4e5).
 * Calls on one handle must be ordered by the stream and must not overlap: the handle's workspace
 * carries state from one call to the next.  Errors: NE_ERR_ARG, NE_ERR_STATE, NE_ERR_HIP.  After
 * NE_ERR_HIP from a training call (a kernel launch failed part-way through its batches) the handle stays
 * usable: the next training call clears the workspace again before it starts; the tables may hold the
 * batches that were enqueued before the failure and part of the failing one.
 */
ne_status ne_train_batch(ne_tables* tables, const ne_alias* alias, const int32_t* pairs_dev, int64_t B,
                         int32_t K, float lr, uint64_t sample_base, int32_t* neg_out_dev,
                         void* hip_stream);

/*
 * Train on a run of consecutive batches: the n_pairs samples of pairs_dev in batches of B (the last
 * one may be shorter), i.e. ceil(n_pairs / B) iterations of the embedding-training loop of
 * Algorithm 1 on one sample block with one negative-sampling table (Sec. III-C: a GPU trains its
 * vertex embeddings on a sample block against its fixed context partition).  The result is the same
 * as calling ne_train_batch once per batch with lr = lr_host[i] and sample_base + i*B; the call
 * exists because the id-only work of batch i+1 (negative draws, detection of rows named more than
 * once) then runs inside the kernels of batch i: two kernel launches per batch instead of four.
 *   pairs_dev   : device, int32[n_pairs][2]; must stay unchanged until the enqueued work is done.
 *   lr_host     : host, float[ceil(n_pairs / B)], read during the call only.
 *   neg_out_dev : NULL, or device int32[n_pairs][K].
 * Other arguments, semantics and errors as for ne_train_batch.  n_pairs == 0 is a no-op.
 */
ne_status ne_train_block(ne_tables* tables, const ne_alias* alias, const int32_t* pairs_dev,
                         int64_t n_pairs, int64_t B, int32_t K, const float* lr_host,
                         uint64_t sample_base, int32_t* neg_out_dev, void* hip_stream);

/*
 * Train on a sequence of runs, each a run of consecutive batches as in ne_train_block on its own sample
 * block with its own negative-sampling table: what one GPU does over an epoch when it visits its sample
 * blocks one after the other (Sec. III-C, 2D partition of the samples).  Same result as one
 * ne_train_block call per run, in order; the call exists because the id-only work of a run's first batch
 * then rides in the kernels of the previous run's last batch, where separate calls would launch it on its
 * own (two extra kernel launches per run).
 *   runs_host : host, ne_run[n_runs], read during the call only.  Per run: alias (may be NULL if K == 0),
 *               pairs_dev (device, int32[n_pairs][2], 8-byte aligned), n_pairs (0 = the run is skipped),
 *               sample_base (sample index of the run's first pair), neg_out_dev (NULL, or device
 *               int32[n_pairs][K]).  Batches never straddle two runs: the last batch of a run may be short.
 *   lr_host   : host, one float per batch, the runs' batches in order (sum over runs of ceil(n_pairs / B)).
 * Other arguments, semantics and errors as for ne_train_block.  n_runs == 0 is a no-op.
 */
typedef struct ne_run {
    const ne_alias* alias;
    const int32_t* pairs_dev;
    int64_t n_pairs;
    uint64_t sample_base;
    int32_t* neg_out_dev;
} ne_run;
ne_status ne_train_runs(ne_tables* tables, const ne_run* runs_host, int64_t n_runs, int64_t B, int32_t K,
                        const float* lr_host, void* hip_stream);

/*
 * ne_train_block on samples that stay in pinned host memory (the paper's training pipeline, Sec. IV-A:
 * the host-to-device copy of the next sample batches is hidden behind training).  Same batches, same
 * result as ne_train_block; the pairs of batch i+2 are copied into a ring of three batch buffers by a few
 * helper workgroups inside the launch that trains batch i, so no second stream and no event is involved
 * (copies on a second stream ordered by events, whether memcpys or kernels, were measured to cost 6-25 % of
 * the training rate; riding along costs 3 %).
 *   pairs_host_pinned : host, page-locked, int32[n_pairs][2], 8-byte aligned; must stay valid and
 *                       unchanged until the enqueued work is done.
 *   staging_dev       : device, int32[3][B][2], 16-byte aligned, caller-owned scratch.
 * Other arguments, semantics and errors as for ne_train_block; NE_ERR_ARG also when the host buffer is not
 * page-locked.
 */
ne_status ne_train_block_pinned(ne_tables* tables, const ne_alias* alias, const int32_t* pairs_host_pinned,
                                int64_t n_pairs, int64_t B, int32_t K, const float* lr_host,
                                uint64_t sample_base, int32_t* staging_dev, int32_t* neg_out_dev,
                                void* hip_stream);

/*
 * On-device augmentation (Algorithm 1, "network augmentation"; Sec. IV-A variant that merges the
 * augmentation into a later stage): trains directly on random walks instead of on materialised pairs.
 * walks_dev is int32 [n_walks][walk_len] (device); entry i of a walk is the source of the samples
 * (walk[i], walk[i+j]) for 1 <= j <= window with i + j < walk_len, the earlier node being the source; a
 * sample exists only if both entries are non-negative (pad short walks with -1).  Consecutive groups of
 * walks_per_batch walks form the batches; each batch is one minibatch-synchronous step over all of its
 * samples, exactly as ne_train_batch on the same pairs would be, with lr_host[batch].  The negatives of
 * sample (walk r, entry i, offset j), r counted over the whole call, are drawn for sample index
 *   sample_base + (r * walk_len + i) * window + (j - 1),
 * so the result does not depend on how the walks are split into batches beyond the batching itself.
 * A walk entry's vertex row is gathered once for its `window` samples and its delta written once; where
 * the shape allows, a workgroup takes a whole segment of consecutive entries and does the same for their
 * context rows.  Walks are 4 bytes per entry where pairs are 8 bytes per sample.
 *   neg_out_dev : NULL, or device int32 [n_walks][walk_len][window][K]; rows of samples that do not
 *                 exist are left untouched.
 * Needs the training workspace of ne_create_tables with
 *   walks_per_batch * walk_len * (1 + window * (K + 1)) <= max_batch * (max_negatives + 2).
 * 2 <= walk_len <= 65536, 1 <= window <= 64.  n_walks == 0 is a no-op.
 * Errors: NE_ERR_ARG, NE_ERR_STATE, NE_ERR_HIP.
 */
ne_status ne_train_walks(ne_tables* tables, const ne_alias* alias, const int32_t* walks_dev, int64_t n_walks,
                         int64_t walks_per_batch, int32_t walk_len, int32_t window, int32_t K,
                         const float* lr_host, uint64_t sample_base, int32_t* neg_out_dev, void* hip_stream);

/*
 * Shared-negative step: the formulation the paper cites as related work (Sec. VI-B), where all pairs
 * of a mini-batch share one set of negatives so that scoring and both gradient products become dense
 * matrix products.  Every one of the B pairs is scored against the same N negative context rows;
 * negative terms carry the weight neg_scale:
 *   J = sum_b [ log sigmoid(x_b . c_ctx_b) + neg_scale * sum_n log sigmoid(-x_b . c_n) ]
 * and the tables move by lr * dJ, minibatch-synchronously (pre-batch tables, duplicates summed).
 * Negative n is the alias draw for Philox(key = seed, counter = (batch_index_lo, batch_index_hi, n, 2)).
 * Precision: the positive pair is computed in fp32.  For the dense part the gathered rows are rounded
 * to bfloat16 (nearest even), S = Xq . Cq^T accumulates in fp32 on the matrix cores,
 * G = -neg_scale * sigmoid(S) is formed in fp32 and rounded to bfloat16, and G . Cq and G^T . Xq
 * accumulate in fp32; the tables stay fp32 (rows that one reference of the batch names are rewritten
 * with plain stores, rows named more than once take fp32 atomic adds, so their sums depend on order).
 *   dim must be 64, 128 or 256; 1 <= B <= 2^20; N a multiple of 128 in [128, 65536].
 *   workspace_dev : device scratch, 256-byte aligned, at least ne_shared_workspace_bytes(dim, B, N)
 *                   bytes, overwritten; needs no initialisation and carries nothing between calls.
 *   neg_out_dev   : NULL, or device int32[N] receiving the negative ids.
 *   loss_sum_dev  : NULL, or device double (caller-zeroed) to which the batch's summed loss at the
 *                   pre-batch tables is added: sum_b [softplus(-s_b0) + neg_scale sum_n softplus(S_bn)].
 * B == 0 is a no-op.  Errors: NE_ERR_ARG, NE_ERR_STATE, NE_ERR_HIP.
 */
size_t ne_shared_workspace_bytes(int32_t dim, int64_t B, int32_t N);
ne_status ne_train_batch_shared(ne_tables* tables, const ne_alias* alias, const int32_t* pairs_dev,
                                int64_t B, int32_t N, float lr, float neg_scale, uint64_t batch_index,
                                void* workspace_dev, size_t workspace_bytes, int32_t* neg_out_dev,
                                double* loss_sum_dev, void* hip_stream);

/*
 * ne_train_batch_shared for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (minus
 * the workspace), same kernels, same result.  The scratch is a static device array of
 * NE_SHARED_STATIC_SCRATCH_BYTES (32 MiB) inside the library, one per GPU, held from the moment the
 * library's code is loaded on that GPU until the process ends; its address is looked up on the first
 * call on each device.  The call allocates and frees nothing.
 *   Limit: ne_shared_workspace_bytes(dim, B, N) <= NE_SHARED_STATIC_SCRATCH_BYTES (for example dim 256
 *   with B <= 3072 and N <= 1024, or dim 128 with B <= 6144 and N <= 1024); larger shapes return
 *   NE_ERR_ARG and a message that names both sizes.
 *   All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams, two
 *   host threads) race and give wrong results; order them on one stream.  Nothing in the array has to
 *   survive from one call to the next, and nothing in it has to start at zero: every call rewrites what
 *   it reads.
 * Errors: as ne_train_batch_shared, and NE_ERR_HIP if the array's address cannot be obtained.
 */
enum { NE_SHARED_STATIC_SCRATCH_BYTES = 32 * 1024 * 1024 };
ne_status ne_train_batch_shared_static(ne_tables* tables, const ne_alias* alias, const int32_t* pairs_dev,
                                       int64_t B, int32_t N, float lr, float neg_scale, uint64_t batch_index,
                                       int32_t* neg_out_dev, double* loss_sum_dev, void* hip_stream);

/*
 * Per-sample ("asynchronous") training: the loop of Algorithm 1 taken pair by pair instead of batch by
 * batch, as far as a parallel machine can.  The arithmetic per pair is that of ne_train_batch, and no
 * update is ever lost, but the pairs of a call do not wait for each other:
 *   - a row that only one reference of the call names is read and rewritten by that reference alone
 *     (old + delta, plain stores), exactly as in ne_train_batch;
 *   - a row that several references of the call name receives each of their deltas as fp32 atomic adds on
 *     the table row itself, at the moment the reference has computed it.  Every delta arrives, so the row
 *     ends at old + the sum of all deltas; but a pair that reads the row may see it before, after or half-way
 *     through another pair's addition.  Gradients of such pairs are therefore evaluated at a mixture of the
 *     values before the call and values already updated inside it, where ne_train_batch uses the values
 *     before the call for all of them and a sequential loop the fully updated ones.
 * The result depends on timing wherever rows are shared inside a call and is not reproducible bit for bit;
 * it equals ne_train_batch (up to fp32 rounding) when no row is named twice in the call.  No delta slots,
 * no second pass over the shared rows: the call costs the train kernel plus a small id-only launch per batch.
 * ne_train_block_async takes a run of batches like ne_train_block (the id-only work of batch i+1 rides in
 * the kernels of batch i); ne_train_batch_async is one batch.  Both need the training workspace of
 * ne_create_tables (they find out which rows are shared the way ne_train_batch does).
 * Negatives, arguments and errors as for ne_train_block / ne_train_batch.
 */
ne_status ne_train_block_async(ne_tables* tables, const ne_alias* alias, const int32_t* pairs_dev,
                               int64_t n_pairs, int64_t B, int32_t K, const float* lr_host,
                               uint64_t sample_base, int32_t* neg_out_dev, void* hip_stream);
ne_status ne_train_batch_async(ne_tables* tables, const ne_alias* alias, const int32_t* pairs_dev,
                               int64_t B, int32_t K, float lr, uint64_t sample_base,
                               int32_t* neg_out_dev, void* hip_stream);

/*
 * Loss of a batch at the current tables with the same negatives ne_train_batch would draw; nothing
 * is updated.  Adds  sum_b [ -log sigmoid(s_b0) - sum_k log sigmoid(-s_bk) ]  (fp32 terms, fp64 sum)
 * to *loss_sum_dev.
 *   loss_sum_dev : device double, caller-zeroed, read back by the caller after syncing the stream.
 *   neg_out_dev  : NULL, or device int32[B][K] that receives the negative ids.
 * Errors: NE_ERR_ARG, NE_ERR_STATE, NE_ERR_HIP.
 */
ne_status ne_eval_loss(const ne_tables* tables, const ne_alias* alias, const int32_t* pairs_dev,
                       int64_t B, int32_t K, uint64_t sample_base, double* loss_sum_dev,
                       int32_t* neg_out_dev, void* hip_stream);

/*
 * Sub-part training (Sec. III-B: a GPU's vertex embeddings are split into k sub-parts; one is trained
 * while the others travel between host and device through ping-pong buffers).  Tells the handle that
 * vertex rows [first_row, first_row + num_rows) now live at vertex_window_dev (fp32 [num_rows][dim],
 * device, 16-byte aligned, caller-owned); every later call on the handle must only name source ids
 * inside that window (ids outside it are undefined behaviour, as out-of-range ids are).  The context
 * table is unaffected.  Host-side only: nothing is enqueued, so the caller orders the switch against
 * its own copies with streams and events.  Errors: NE_ERR_ARG.
 */
ne_status ne_set_vertex_window(ne_tables* tables, float* vertex_window_dev, int64_t first_row,
                               int64_t num_rows);

/*
 * Evaluation helper (link prediction, Sec. V-B): the similarity score of arbitrary node pairs at the
 * current tables,  scores_dev[i] = vertex[pairs[i][0]] . second[pairs[i][1]]  in fp32, where second is
 * the context table (second_from_context != 0: the score the training objective uses) or the vertex
 * table (0).  pairs_dev int32[n][2] and scores_dev float[n] are device buffers of the caller; ids are
 * not range-checked.  The tables are only read.  n == 0 is a no-op.  Errors: NE_ERR_ARG, NE_ERR_HIP.
 */
ne_status ne_score_pairs(const ne_tables* tables, const int32_t* pairs_dev, int64_t n,
                         int32_t second_from_context, float* scores_dev, void* hip_stream);

/*
 * Tuning of the exact step (ne_train_batch, ne_train_block, ne_train_block_pinned, ne_train_walks); the
 * results are the same sums either way.  The paper fixes neither choice (it never describes its kernel).
 *   list_cap          how a row that several references of a batch name ("shared row") collects
 *                     their deltas: its first list_cap
 *                     references (0..8) store them with plain stores, one buffer row per reference,
 *                     and the rest add to the row's accumulator with atomics.  0 = atomics only.
 *                     -1 = automatic: 8 when the tables are small next to the batch
 *                     (num_nodes <= min(20, 1500 / dim) * rows named per batch), else 0.
 *   sweep_per_thread  hash positions each thread of the apply kernel sweeps: 2, 4 or 8; 0 = automatic
 *                     (2 with the list path, else 4).
 * Takes effect from the next training call on this handle.  Errors: NE_ERR_ARG.
 */
ne_status ne_set_tuning(ne_tables* tables, int32_t list_cap, int32_t sweep_per_thread);

/*
 * Debug helper for the sample format of Table I: counts ids in pairs_dev int32[B][2] that fall
 * outside [0, num_nodes) and adds the count to *bad_count_dev (device uint64, caller-zeroed).
 */
ne_status ne_validate_pairs(const ne_tables* tables, const int32_t* pairs_dev, int64_t B,
                            unsigned long long* bad_count_dev, void* hip_stream);

/*
 * Debug helper: the home position the exact step's duplicate detection gives a row key in a table of
 * `positions` hash positions (a power of two in [2, 2^31]; 0xFFFFFFFF is returned otherwise): the top
 * log2(positions) bits of key * 0x9E3779B1 mod 2^32.  key = row id, with bit 31 set for context rows.
 * A batch uses the smallest power of two >= max(2048, 2 * references) positions, references = B * (K + 2)
 * <= 2^28, so at most 2^29.  Host-only; exists so that the spread of home positions can be checked
 * without a GPU.
 */
uint32_t ne_hash_position(uint32_t key, uint32_t positions);

/*
 * Measurement hooks (instrumentation for benchmarks, not part of the method).  After
 * ne_profile_enable(t, n, max_samples) with n > 0, every n-th ne_train_batch call records a HIP event
 * on the stream immediately before and after its train kernel (the kernel that gathers the rows,
 * scores and writes them back; for ne_train_batch_shared: the scores kernel with the S and dX
 * products), for at most max_samples (<= 65536) calls; n = 0 switches it off.
 * Two events are recorded back to back before the kernel; the gap between them is taken as the cost
 * of recording and subtracted.  ne_profile_read waits for the recorded events, stores the sum of
 * the kernel durations in milliseconds in *total_ms_host and their number in *samples_host (both
 * host), and starts over.
 */
ne_status ne_profile_enable(ne_tables* tables, int32_t every_n, int32_t max_samples);
ne_status ne_profile_read(ne_tables* tables, double* total_ms_host, int64_t* samples_host);

void ne_destroy_tables(ne_tables* tables);
void ne_destroy_alias(ne_alias* alias);

/* Message for the last non-NE_OK status returned on the calling thread (valid until the next call). */
const char* ne_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* NE_H */
