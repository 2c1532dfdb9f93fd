/*
 * gs.h -- C boundary of the random-walk + skip-gram (SGNS) node-embedding path
 * for AMD gfx950.
 *
 * The calls follow the statement of the problem in GraphScale (arXiv
 * 2407.15452): a trainer that holds the whole graph topology (Sec. 3.1),
 * samples random walks from its source nodes and turns them into positive and
 * negative samples (Sec. 2.2, Sec. 3.2), and then reads, and writes back, only
 * the rows of the N x d embedding matrices that the batch names (Sec. 3.2),
 * with a barrier after the write (Sec. 3.2, "Synchronization").
 *
 * Conventions shared by every call
 *  - Every pointer is a DEVICE pointer unless its comment says "host".  The
 *    gs_csr / gs_alias descriptors themselves are small host structs that hold
 *    device pointers.  The caller owns all memory; the library allocates
 *    nothing that outlives a call and frees nothing.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls only enqueue work; outputs, including the scalar outputs written
 *    through device pointers, are valid once the stream has been synchronised.
 *  - Calls that need scratch memory take (ws, ws_bytes); the matching
 *    *_workspace_bytes() function (host, O(1)) returns the size to provide.
 *    ws must be 256-byte aligned.  Its contents are undefined afterwards.
 *  - Return value: GS_OK or a negative gs_status.  Arguments are validated on
 *    the host only; nothing is enqueued when a call fails validation.  Node
 *    ids live in device memory and are checked by the kernels that use them as
 *    row numbers: edge lists drop them, walks stop at them (`starts`, CSR
 *    neighbours), the training steps read row 0 instead and report a NaN loss,
 *    the storage operations skip them.  CSR offsets and the alias[] entries of
 *    a table are trusted as built by gs_csr_build / gs_alias_build.
 *  - Node ids are int32.  CSR offsets are int32 or int64 (`offset_bits`).
 *  - Random numbers are Philox4x32-10 blocks keyed by the caller's 64-bit
 *    seed; the counter is (index low, index high, c2, c3) as stated per call,
 *    so any sub-range of walks or pairs can be produced on its own and is
 *    identical to the same range of one big call.
 *  - slot(r, n) = high 64 bits of the 128-bit product r * n, r = (word0 << 32)
 *    | word1;  unit(x) = (float)(x >> 8) * 2^-24.
 */
#ifndef GS_H_
#define GS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  GS_OK = 0,
  GS_EINVAL = -1,     /* null / negative / misaligned / unsupported argument      */
  GS_EWORKSPACE = -2, /* ws_bytes smaller than *_workspace_bytes() reports        */
  GS_EOVERFLOW = -3,  /* a count does not fit the chosen index type               */
  GS_EHIP = -4        /* a HIP runtime call failed; see gs_last_hip_error()       */
} gs_status;

enum { GS_SYMMETRIZE = 1, GS_DROP_SELF_LOOPS = 2, GS_DEDUPE = 4 };
enum { GS_F32 = 0, GS_BF16 = 1, GS_F16 = 2 };  /* table storage: float, bfloat16, IEEE binary16 */

/* Graph topology in CSR form; every row sorted ascending by neighbour id. */
typedef struct {
  int64_t num_nodes;
  int64_t num_entries;   /* directed entries; an undirected edge is two        */
  const void* offsets;   /* int32[num_nodes+1] or int64[num_nodes+1]           */
  int32_t offset_bits;   /* 32 or 64                                            */
  const int32_t* nbrs;   /* int32[num_entries]                                  */
  const float* weights;  /* float[num_entries] or NULL (unused by the walkers) */
} gs_csr;

/* Alias table(s).  For walks: one table per CSR row, stored at the row's
 * offsets, alias[] = position inside the row.  For negatives: one table of
 * num_nodes entries.  prob == NULL means "uniform".  `packed` is optional
 * (NULL: not provided): the same table with entry i stored as one 8-byte word,
 * prob bits in the low half and alias in the high half, as written by
 * gs_alias_pack; the samplers read it instead of the two arrays when present
 * (one random cache line per draw instead of two). */
typedef struct {
  const float* prob;
  const int32_t* alias;
  const uint64_t* packed;
} gs_alias;

/* HIP error code of the last GS_EHIP on this thread (0 if none). */
int32_t gs_last_hip_error(void);

/* --------------------------------------------------------------------------
 * gs_csr_build -- edge list to CSR (Sec. 3.1: the topology a trainer keeps).
 *   src, dst  int32[m]; w float[m] or NULL.
 *   Edges with an endpoint outside [0, num_nodes) are dropped.  flags:
 *   GS_DROP_SELF_LOOPS drops src == dst; GS_SYMMETRIZE also inserts the
 *   reverse of every edge; GS_DEDUPE keeps one entry per (src, dst), the one
 *   from the lowest input index (its weight is kept).  Rows come out sorted by
 *   neighbour id, equal neighbours in input order.
 *   offsets_out  int32|int64 [num_nodes+1];  nbrs_out int32[cap], w_out
 *   float[cap] (required iff w != NULL), cap = m, or 2m with GS_SYMMETRIZE;
 *   num_entries_out  int64[1] on the device.
 *   Errors: GS_EOVERFLOW if offset_bits == 32 and cap > INT32_MAX, or
 *   m >= 2^31.
 * ------------------------------------------------------------------------ */
size_t gs_csr_build_workspace_bytes(int64_t m, int64_t num_nodes, uint32_t flags);
int32_t gs_csr_build(const int32_t* src, const int32_t* dst, const float* w, int64_t m,
                     int64_t num_nodes, uint32_t flags, int32_t offset_bits,
                     void* offsets_out, int32_t* nbrs_out, float* w_out,
                     int64_t* num_entries_out, void* ws, size_t ws_bytes, void* stream);

/* --------------------------------------------------------------------------
 * gs_alias_build -- alias tables for weighted draws: per-row tables for
 * weighted walks, or one table over degree^0.75 for the negatives of Sec. 2.2
 * (the weights are an input; the library does not compute powers).
 *   seg_offsets int32|int64 [num_segments+1]; segment s covers
 *   weights[seg_offsets[s] .. seg_offsets[s+1]);  total_entries =
 *   seg_offsets[num_segments] (host value, used for sizing only).
 *   Construction (per segment, n entries, fp64 inside): S = sum of weights in
 *   index order; mass_i = w_i * n; entries with mass < S are "small", others
 *   "large", both first-in first-out in index order; repeatedly the oldest
 *   small a and oldest large b give prob[a] = (float)(mass_a / S), alias[a] =
 *   b, mass_b = (mass_b + mass_a) - S, and b is appended to the list its new
 *   mass selects; leftovers get prob = 1, alias = self.  alias[] is a position
 *   inside the segment.  Segments longer than INT32_MAX are unsupported.
 * ------------------------------------------------------------------------ */
size_t gs_alias_build_workspace_bytes(int64_t num_segments, int64_t total_entries);
int32_t gs_alias_build(const void* seg_offsets, int32_t offset_bits, int64_t num_segments,
                       int64_t total_entries, const float* weights, float* prob_out,
                       int32_t* alias_out, void* ws, size_t ws_bytes, void* stream);

/* gs_alias_pack -- interleaves a finished table for the samplers:
 *   packed_out[i] = (uint64)alias[i] << 32 | bits(prob[i]),  i in [0, total_entries). */
int32_t gs_alias_pack(const float* prob, const int32_t* alias, int64_t total_entries,
                      uint64_t* packed_out, void* stream);

/* --------------------------------------------------------------------------
 * gs_random_walk -- first-order walks (Sec. 2.2, DeepWalk; Sec. 3.2 counts
 * walk_len sampled NODES per source, so a walk makes walk_len - 1 steps).
 *   g, a: host structs (a == NULL or a->prob == NULL: uniform neighbour).
 *   starts int32[num_walks]; walks_out int32[num_walks][walk_len], row-major.
 *   Step t of walk id = walk_id_base + i uses the Philox block with counter
 *   (id low, id high, t, 0): neighbour slot(r, deg); if weighted and not
 *   unit(word2) < prob[slot], alias[slot] instead.  A node without out-edges
 *   (or a start outside [0, num_nodes)) ends the walk: the rest of the row is -1.
 * ------------------------------------------------------------------------ */
int32_t gs_random_walk(const gs_csr* g, const gs_alias* a, const int32_t* starts,
                       int64_t num_walks, uint64_t walk_id_base, int32_t walk_len,
                       uint64_t seed, int32_t* walks_out, void* stream);

/* --------------------------------------------------------------------------
 * gs_node2vec_walk -- second-order biased walks (Sec. 2.2, node2vec).
 *   As gs_random_walk, but from the second step on a candidate x drawn from
 *   the row of the current node is accepted with probability bias / max_bias:
 *   bias = 1/p if x is the previous node, 1 if the previous node has an edge
 *   to x, 1/q otherwise; max_bias = max(1/p, 1, 1/q) (all fp32, computed on
 *   the host).  Attempt `att` of step t uses counter (id low, id high, t,
 *   att); accept iff unit(word3) * max_bias < bias.  att runs 0..1023 and the
 *   candidate of attempt 1023 is taken unconditionally.
 *   Errors: GS_EINVAL unless p > 0 and q > 0.
 * ------------------------------------------------------------------------ */
int32_t gs_node2vec_walk(const gs_csr* g, const gs_alias* a, const int32_t* starts,
                         int64_t num_walks, uint64_t walk_id_base, int32_t walk_len,
                         float p, float q, uint64_t seed, int32_t* walks_out, void* stream);

/* --------------------------------------------------------------------------
 * gs_make_pairs -- skip-gram (centre, context) pairs of Sec. 2.2 with the
 * paper's "window-size".
 *   walks int32[num_walks][walk_len] (-1 only as a suffix).  For walk i, then
 *   position a of its valid prefix, then offset b = -window..window, b != 0,
 *   with a + b inside the prefix: (walks[i][a], walks[i][a+b]).  Dense output
 *   in that order; capacity of centers_out / contexts_out:
 *   num_walks * (2*window*walk_len - window*(window+1)) entries when walk_len
 *   > window, num_walks * walk_len * (walk_len - 1) otherwise.
 *   num_pairs_out int64[1] on the device.  walk_len <= 4096.
 * ------------------------------------------------------------------------ */
size_t gs_make_pairs_workspace_bytes(int64_t num_walks);
int32_t gs_make_pairs(const int32_t* walks, int64_t num_walks, int32_t walk_len, int32_t window,
                      int32_t* centers_out, int32_t* contexts_out, int64_t* num_pairs_out,
                      void* ws, size_t ws_bytes, void* stream);

/* --------------------------------------------------------------------------
 * gs_sample_negatives -- the "negatively sampled nodes" of Sec. 3.2.
 *   negs_out int32[num_pairs][k].  Entry (i, j) is an alias draw from the
 *   single table `noise` of num_nodes entries with counter (idx low, idx
 *   high, j, 0x80000000), idx = pair_index_base + i.  Draws are independent;
 *   a negative equal to the centre or context is kept.
 * ------------------------------------------------------------------------ */
int32_t gs_sample_negatives(const gs_alias* noise, int64_t num_nodes, int64_t num_pairs,
                            uint64_t pair_index_base, int32_t k, uint64_t seed,
                            int32_t* negs_out, void* stream);

/* --------------------------------------------------------------------------
 * gs_sample_edges -- the positive pairs of a LINE batch (Sec. 3.2: a LINE batch
 * of B source nodes holds B * (2 + num_neg) nodes; Sec. 4 trains LINE with 5
 * negatives per source node).  Sample i draws one CSR entry e, uniformly when
 * edge_alias is NULL or has prob == NULL, otherwise as an alias draw from one
 * table over all g->num_entries entries (gs_alias_build with the single
 * segment {0, num_entries} over the entry weights; alias[] = entry index),
 * with counter (idx low, idx high, 0, 0x40000000), idx = sample_index_base +
 * i, and returns centers_out[i] = the row that holds e, contexts_out[i] =
 * nbrs[e].  In a symmetrised graph both directions of an edge are entries.
 * The batch is then an ordinary gs_sgns_step batch (second-order proximity:
 * source rows in w_in, context rows in w_out) or a gs_line1_step batch
 * (first-order proximity, one table), with negatives from gs_sample_negatives.
 *   centers_out, contexts_out  int32[num_samples] on the device.
 *   Errors: GS_EINVAL for an empty graph (num_entries < 1), offset_bits other
 *   than 32 / 64, or a prob without alias.
 * ------------------------------------------------------------------------ */
int32_t gs_sample_edges(const gs_csr* g, const gs_alias* edge_alias, int64_t num_samples,
                        uint64_t sample_index_base, uint64_t seed, int32_t* centers_out,
                        int32_t* contexts_out, void* stream);

/* --------------------------------------------------------------------------
 * gs_sgns_step -- one training iteration of Sec. 3.2: fetch the batch's rows,
 * loss and sparse gradient on them, write those rows back; reads see the
 * tables as they were before the call (the barrier of "Synchronization").
 *   w_in, w_out  [num_nodes][dim] row-major, float (GS_F32), bfloat16 (GS_BF16)
 *   or IEEE binary16 (GS_F16; Sec. 4.2 keeps the industry-scale table in fp16);
 *   the 16-bit formats are widened exactly and computed on in fp32.  Updated in
 *   place.
 *   For pair i: u = w_in[centers[i]], v_0 = w_out[contexts[i]], v_j =
 *   w_out[negs[i][j-1]], x_j = <u, v_j>; loss_i = softplus(-x_0) + sum_j
 *   softplus(x_j); g_0 = sigmoid(x_0) - 1, g_j = sigmoid(x_j);
 *   w_in[c] -= lr * sum g_j v_j;  w_out[row_j] -= lr * g_j u, summed over all
 *   occurrences in the batch.  loss_sum_out double[1] on the device receives
 *   the sum of loss_i (overwritten).
 *   Every touched element is written once, as round(old + delta) with delta
 *   the exact sum of the fp32 products (16-bit formats: round to nearest even
 *   through fp32).
 *   dim must be a multiple of 4 (fp32) or 8 (16-bit) and at most 1024; k <= 60;
 *   num_pairs * (k+1) < 2^31.  Rows that the batch does not name are not
 *   touched.  w_in and w_out must be two tables (GS_EINVAL if they are the
 *   same address).  The ids live on the device and are checked there: an id
 *   outside [0, num_nodes) is treated as row 0, so no access leaves the
 *   tables, and loss_sum_out is set to NaN to report it (the tables are then
 *   not meaningful).  The same report is made when a product lr * element
 *   reaches 16384 in magnitude (the exact accumulation of the row sums covers
 *   products below 32768).  The row sums are exact (64-bit fixed point, multiples
 *   of 2^-36), so the same call on the same inputs gives the same bits every
 *   time.  The workspace holds the per-term coefficients, the terms regrouped by
 *   destination row, a counter per key (two per node, or per key of the batch
 *   when the graph is much larger than the batch), a side buffer for rows with
 *   many terms and the staged centre-row gradients.
 * ------------------------------------------------------------------------ */
size_t gs_sgns_step_workspace_bytes(int64_t num_pairs, int64_t num_nodes, int32_t k, int32_t dim,
                                    int32_t dtype);
int32_t gs_sgns_step(void* w_in, void* w_out, int64_t num_nodes, int32_t dim, int32_t dtype,
                     const int32_t* centers, const int32_t* contexts, const int32_t* negs,
                     int64_t num_pairs, int32_t k, float lr, double* loss_sum_out,
                     void* ws, size_t ws_bytes, void* stream);

/* --------------------------------------------------------------------------
 * gs_sgns_step_static -- gs_sgns_step for callers that cannot allocate or hand
 * over device memory for a workspace: code under HIP graph capture, tight
 * training or serving loops, harnesses that forbid hipMalloc.  The scratch memory
 * of the step is a 12 MiB array that is part of the library's code object on
 * every GPU (held until the process ends); the call allocates and frees nothing.
 *   Same arguments (without ws, ws_bytes), results and errors as gs_sgns_step,
 *   for small batches: num_pairs <= 4096, num_pairs * (k+1) <= 65536, dim <=
 *   256; GS_EWORKSPACE beyond that.  The graph may have any size (the step
 *   counts over a table of the batch's keys).
 *   All calls on one GPU share that GPU's array: calls that overlap in time on
 *   one GPU (two streams, two threads) race; one call at a time per GPU.  The
 *   first call on a device looks the array's address up (hipGetSymbolAddress)
 *   and should therefore be made outside a graph capture.
 * ------------------------------------------------------------------------ */
int32_t gs_sgns_step_static(void* w_in, void* w_out, int64_t num_nodes, int32_t dim, int32_t dtype,
                            const int32_t* centers, const int32_t* contexts, const int32_t* negs,
                            int64_t num_pairs, int32_t k, float lr, double* loss_sum_out,
                            void* stream);

/* --------------------------------------------------------------------------
 * gs_sgns_momentum_step -- the same iteration with the optimizer the paper
 * runs: SGD with momentum written as the three storage operations of Sec. 3.2
 * (model update for SGD with momentum), applied to both tables:
 *     mult      momentum <- mu * momentum                 every row
 *     put       momentum[r] <- momentum[r] + gradient[r]  rows the batch names
 *     mult_add  model <- model - lr * momentum            every row
 *   gradient = gradient of the batch's summed loss at the pre-iteration model
 *   (the same terms gs_sgns_step applies).  m_in, m_out: momentum tables, same
 *   shape and dtype as w_in, w_out, distinct from them, updated in place.
 *   Unlike gs_sgns_step this streams over all four tables once or twice per
 *   call (two dense passes), as the paper's formulation does.
 *   Workspace: gs_sgns_step_workspace_bytes().  Other arguments and errors as
 *   for gs_sgns_step.
 * ------------------------------------------------------------------------ */
int32_t gs_sgns_momentum_step(void* w_in, void* w_out, void* m_in, void* m_out, int64_t num_nodes,
                              int32_t dim, int32_t dtype, const int32_t* centers,
                              const int32_t* contexts, const int32_t* negs, int64_t num_pairs,
                              int32_t k, float lr, float mu, double* loss_sum_out, void* ws,
                              size_t ws_bytes, void* stream);

/* --------------------------------------------------------------------------
 * gs_sgns_step_fused -- gs_sample_negatives and gs_sgns_step in one call: the
 * negatives of pair i are drawn inside the step, from the same counters
 * (pair_index_base + i, j, 0x80000000) and the same table `noise` (NULL or
 * prob == NULL: uniform over the nodes), so the result is that of the two
 * calls; the caller provides no negs array (the draws are kept in the
 * workspace for the later kernels of the step).
 *   Other arguments, limits and errors as for gs_sgns_step; the workspace is
 *   gs_sgns_step_fused_workspace_bytes (the step's own plus 4*num_pairs*k).
 * ------------------------------------------------------------------------ */
size_t gs_sgns_step_fused_workspace_bytes(int64_t num_pairs, int64_t num_nodes, int32_t k,
                                          int32_t dim, int32_t dtype);
int32_t gs_sgns_step_fused(void* w_in, void* w_out, int64_t num_nodes, int32_t dim, int32_t dtype,
                           const int32_t* centers, const int32_t* contexts, int64_t num_pairs,
                           const gs_alias* noise, uint64_t pair_index_base, uint64_t neg_seed,
                           int32_t k, float lr, double* loss_sum_out, void* ws, size_t ws_bytes,
                           void* stream);

/* --------------------------------------------------------------------------
 * gs_pair_offsets, gs_sgns_step_from_walks -- sampling and update in one call
 * (Sec. 2.2: walks -> skip-gram pairs -> negative sampling; Sec. 3.2: the
 * sampled nodes of a batch are fetched and trained on): the iteration derives
 * its (centre, context) pairs from the walk buffer and draws its negatives
 * inside the forward kernel, so no centers / contexts / negs arrays exist at
 * the boundary (the derived ids are kept in the workspace for the later kernels
 * of the step).
 *
 * gs_pair_offsets: offsets_out int64[num_walks+1]; offsets_out[w] = number of
 *   pairs gs_make_pairs emits for the walks before w, offsets_out[num_walks] =
 *   for all of them.  Once per walk buffer.
 *
 * gs_sgns_step_from_walks: the batch is pairs first_pair .. first_pair +
 *   num_pairs - 1 of the sequence gs_make_pairs would emit for walks[0 ..
 *   num_walks) (any slice: batch boundaries need not fall on walks); negative j
 *   of pair i is the draw of gs_sample_negatives for pair index pair_index_base
 *   + i.  The result is that of gs_make_pairs + gs_sample_negatives +
 *   gs_sgns_step on that slice.  If the walks hold fewer than first_pair +
 *   num_pairs pairs, or pair_offsets is not the numbering of these walks,
 *   loss_sum_out is NaN (as for an id that is no row; no access leaves the
 *   walk buffer).
 *   walks int32[num_walks][walk_len]; pair_offsets as written by gs_pair_offsets;
 *   other arguments, limits and errors as for gs_sgns_step_fused; workspace
 *   gs_sgns_step_from_walks_workspace_bytes.
 * ------------------------------------------------------------------------ */
size_t gs_pair_offsets_workspace_bytes(int64_t num_walks);
int32_t gs_pair_offsets(const int32_t* walks, int64_t num_walks, int32_t walk_len, int32_t window,
                        int64_t* offsets_out, void* ws, size_t ws_bytes, void* stream);
size_t gs_sgns_step_from_walks_workspace_bytes(int64_t num_pairs, int64_t num_nodes, int32_t k,
                                               int32_t dim, int32_t dtype);
int32_t gs_sgns_step_from_walks(void* w_in, void* w_out, int64_t num_nodes, int32_t dim, int32_t dtype,
                                const int32_t* walks, int64_t num_walks, int32_t walk_len,
                                int32_t window, const int64_t* pair_offsets, int64_t first_pair,
                                int64_t num_pairs, const gs_alias* noise, uint64_t pair_index_base,
                                uint64_t neg_seed, int32_t k, float lr, double* loss_sum_out, void* ws,
                                size_t ws_bytes, void* stream);

/* --------------------------------------------------------------------------
 * gs_line1_step -- LINE iteration with first-order proximity (the LINE variant
 * with one embedding per node; Sec. 2.2 / Sec. 4 cite LINE, Sec. 3.2 gives the
 * batch shape): one table w on both sides.  For pair i: u = w[sources[i]],
 * v_0 = w[targets[i]], v_j = w[negs[i][j-1]]; loss and g_j as in gs_sgns_step;
 * w[sources[i]] gets -lr * sum_j g_j v_j and w[row_j] gets -lr * g_j u, all
 * from the values before the call.  A row is written as round(old + delta)
 * once for what it receives as target / negative and then once more for what it
 * receives as source (two roundings for a row that is both).
 *   Arguments, limits, id checking and errors as for gs_sgns_step; workspace
 *   gs_line1_step_workspace_bytes (the step's own plus a copy of one input row
 *   and 4 bytes per pair).
 * ------------------------------------------------------------------------ */
size_t gs_line1_step_workspace_bytes(int64_t num_pairs, int64_t num_nodes, int32_t k, int32_t dim,
                                     int32_t dtype);
int32_t gs_line1_step(void* w, int64_t num_nodes, int32_t dim, int32_t dtype, const int32_t* sources,
                      const int32_t* targets, const int32_t* negs, int64_t num_pairs, int32_t k,
                      float lr, double* loss_sum_out, void* ws, size_t ws_bytes, void* stream);

/* --------------------------------------------------------------------------
 * gs_sgns_adam_step -- the iteration with Adam kept inside the storage (Sec. 3.2
 * names Adam next to SGD with momentum; the rule is Kingma & Ba's), run like
 * the momentum step as dense operations around a sparse put of the batch's
 * gradient rows g (gradient of the summed loss at the pre-iteration model):
 *   mult   m <- beta1 * m, v <- beta2 * v                         (every row)
 *   put    m[r] += (1 - beta1) * g[r], v[r] += (1 - beta2) * g[r]^2  (batch rows)
 *   apply  w <- w - (lr / (1 - beta1^t)) * m / (sqrt(v) / sqrt(1 - beta2^t) + eps)
 * for both tables; t >= 1 is the number of this iteration.  Six distinct fp32
 * tables [num_nodes][dim], 16-byte aligned; other arguments, workspace and
 * limits as for gs_sgns_step with dtype GS_F32.
 *   Errors: GS_EINVAL also for t < 1, beta outside [0, 1), eps < 0, or two
 *   tables at the same address.
 * ------------------------------------------------------------------------ */
int32_t gs_sgns_adam_step(float* w_in, float* w_out, float* m_in, float* m_out, float* v_in,
                          float* v_out, int64_t num_nodes, int32_t dim, const int32_t* centers,
                          const int32_t* contexts, const int32_t* negs, int64_t num_pairs, int32_t k,
                          float lr, float beta1, float beta2, float eps, int64_t t,
                          double* loss_sum_out, void* ws, size_t ws_bytes, void* stream);

/* --------------------------------------------------------------------------
 * Storage operations on a batch of vertex ids (Sec. 3.1: a trainer merges equal
 * vertex ids before it makes a single request and gets one block of rows back;
 * Sec. 3.2: only the n << N rows of a mini-batch are fetched, and only an
 * n x d block of gradient rows is sent back and added to the storage).
 *
 * gs_unique_ids -- distinct ids of the batch in ascending order.
 *   ids int32[n] (n < 2^31).  unique_out int32[n] (the first *num_unique_out
 *   entries are written), num_unique_out int64[1] on the device, inverse_out
 *   int32[n] or NULL: position of ids[i] in unique_out.  Ids outside
 *   [0, num_nodes) are left out of unique_out and get inverse -1.
 *   Workspace: gs_unique_ids_workspace_bytes(n, num_nodes) (a bitmap of the node
 *   ids, or sort buffers for the batch when the graph is far larger).
 *
 * gs_get_rows -- out[i] = table[ids[i]] for i < n, as fp32 (bf16 rows widened
 *   exactly); a zero row for an id outside [0, num_nodes).  out float[n][dim].
 *
 * gs_put_rows -- table[ids[i]] = round(table[ids[i]] + scale * rows[i]), one
 *   rounding per element (fp32 tables: of the exact sum to fp64 then fp32; bf16
 *   tables: from there to bf16, nearest even).  rows float[n][dim].  The ids
 *   must be distinct (as gs_unique_ids returns them): rows of equal ids race.
 *   Ids outside [0, num_nodes) are skipped.
 *
 *   count_dev (both calls): NULL, or int64[1] on the device: only the first
 *   min(n, *count_dev) ids are processed, so that the count written by
 *   gs_unique_ids can be used without a host round trip.
 *   table [num_nodes][dim] of dtype GS_F32 | GS_BF16, 16-byte aligned; dim a
 *   multiple of 4 (fp32) or 8 (bf16).  Errors: GS_EINVAL otherwise.
 * ------------------------------------------------------------------------ */
size_t gs_unique_ids_workspace_bytes(int64_t n, int64_t num_nodes);
int32_t gs_unique_ids(const int32_t* ids, int64_t n, int64_t num_nodes, int32_t* unique_out,
                      int64_t* num_unique_out, int32_t* inverse_out, void* ws, size_t ws_bytes,
                      void* stream);
int32_t gs_get_rows(const void* table, int64_t num_nodes, int32_t dim, int32_t dtype,
                    const int32_t* ids, int64_t n, const int64_t* count_dev, float* out,
                    void* stream);
int32_t gs_put_rows(void* table, int64_t num_nodes, int32_t dim, int32_t dtype, const int32_t* ids,
                    int64_t n, const int64_t* count_dev, const float* rows, float scale,
                    void* stream);

/* --------------------------------------------------------------------------
 * gs_sort_pairs -- reorders a batch of (centre, context) pairs by centre id,
 * keeping the input order among equal centres (stable).  An iteration sums
 * over its batch, so the order of the pairs does not change its result; with
 * equal centres next to each other gs_sgns_step / gs_line1_step load and write
 * each centre row once per run.  Walk batches (gs_make_pairs) already come in
 * runs; a LINE batch (gs_sample_edges) does not.  Ids outside [0, num_nodes)
 * go last, in input order.
 *   centers, contexts int32[n] (n < 2^31); outputs int32[n], distinct from the
 *   inputs.  Negatives are drawn by position afterwards (gs_sample_negatives).
 * ------------------------------------------------------------------------ */
size_t gs_sort_pairs_workspace_bytes(int64_t n);
int32_t gs_sort_pairs(const int32_t* centers, const int32_t* contexts, int64_t n, int64_t num_nodes,
                      int32_t* centers_out, int32_t* contexts_out, void* ws, size_t ws_bytes,
                      void* stream);

/* --------------------------------------------------------------------------
 * gs_table_mult, gs_table_mult_add -- the two dense storage operations of Sec.
 * 3.2 (model update for SGD with momentum): every element of a table times a
 * factor (the momentum table times the momentum value), and dst <- dst +
 * factor * src for two tables of the same shape (the model minus the learning
 * rate times the momentum).  One rounding per element (bf16: through fp32,
 * nearest even).  Tables [num_nodes][dim], GS_F32 | GS_BF16, 16-byte aligned;
 * dim a multiple of 4 (fp32) or 8 (bf16); dst != src.
 * ------------------------------------------------------------------------ */
int32_t gs_table_mult(void* table, int64_t num_nodes, int32_t dim, int32_t dtype, float factor,
                      void* stream);
int32_t gs_table_mult_add(void* dst, const void* src, int64_t num_nodes, int32_t dim, int32_t dtype,
                          float factor, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* GS_H_ */
