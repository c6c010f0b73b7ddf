/* gco.h -- C ABI of the subgraph-GNN training library for AMD MI355X (gfx950).
 *
 * The library trains, on one GPU, one small graph convolutional network per
 * subgraph of a partitioned graph, for a relaxed quadratic 0/1 objective
 * (Maximum Independent Set, Max-Cut), and reads the result out as a 0/1 vector
 * plus the list of cross-subgraph edges.  It covers stage 1 and stage 2 of the
 * paper's Algorithm 1 ("Parallel Subgraph Training", "Probability
 * Reconstruction") and the inputs of stage 3 (conflict edges); all subgraphs of
 * a graph are trained together as one block-diagonal batch.
 *
 * Conventions
 *  - Every call returns a gco_status; nothing throws or aborts across the ABI.
 *    gco_last_error() gives the text of the last failure on that context.
 *  - Pointers are HOST pointers unless the name says "dev".  The caller owns
 *    every buffer it passes, before and after the call; the library copies.
 *  - Node-indexed arrays are in the caller's ORIGINAL node order.  (Inside, nodes
 *    are stored subgraph by subgraph; that order never shows at this boundary.)
 *  - All device work is enqueued on the stream given at creation; calls that
 *    return host data wait for that stream only.
 *  - A context is not thread-safe.  Same inputs give bit-identical outputs from
 *    run to run (no floating-point atomics are used).
 */
#ifndef GCO_H
#define GCO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gco_ctx gco_ctx;

typedef enum {
  GCO_OK = 0,
  GCO_EINVAL = -1,  /* bad argument or malformed graph                      */
  GCO_ENOMEM = -2,  /* device or host allocation failed                     */
  GCO_ESTATE = -3,  /* call out of order (e.g. train before upload_graph)   */
  GCO_EDEVICE = -4, /* a HIP call failed                                    */
  GCO_ERANGE = -5   /* a size is beyond what the library supports           */
} gco_status;

enum { GCO_PROBLEM_MIS = 0, GCO_PROBLEM_MAXCUT = 1 };
enum { GCO_NORM_SYM = 0, GCO_NORM_MEAN = 1 };
enum { GCO_STORAGE_FP32 = 0, GCO_STORAGE_BF16 = 1 };
enum { GCO_REPAIR_NONE = 0, GCO_REPAIR_LOCAL = 1, GCO_REPAIR_ALL = 2 };

/* Device memory hooks.  alloc returns a device pointer aligned to 256 bytes or
 * NULL; free receives what alloc returned.  Both NULL => hipMalloc / hipFree. */
typedef void* (*gco_alloc_fn)(size_t bytes, void* user);
typedef void (*gco_free_fn)(void* dev_ptr, void* user);

typedef struct {
  int32_t problem;        /* GCO_PROBLEM_*: which quadratic objective (Alg. 1 input "QUBO Q") */
  int32_t num_layers;     /* L in {1,2,3}: L-1 hidden ReLU layers of Eq. 3, then a scalar
                             linear layer feeding the sigmoid of Eq. 4                        */
  int32_t dim;            /* width of the node embedding and of every hidden layer:
                             one of 8, 16, 32, 64, 128                                        */
  int32_t norm;           /* GCO_NORM_MEAN: 1/(|N(i)|+1) as printed in Eq. 3;
                             GCO_NORM_SYM: 1/sqrt((|N(i)|+1)(|N(j)|+1))                        */
  int32_t storage;        /* GCO_STORAGE_FP32: all arithmetic and storage in fp32.
                             GCO_STORAGE_BF16: node features and their gradients are
                             stored in bf16 and multiplied on the matrix cores with fp32
                             accumulation; parameters, Adam state, probabilities and the
                             loss stay fp32 (dim 64 or 128 only)                            */
  int32_t weight_sharing; /* 0: one weight set per subgraph (Alg. 1 stage 1: one net per
                             subgraph); 1: one set shared by all subgraphs                    */
  int32_t train_embed;    /* 1: node embeddings are trained; 0: only W (Sec. 3.2 names W only) */
  float alpha, beta;      /* MIS: L = alpha * sum_{(i,j) in E} p_i p_j - beta * sum_i p_i (Eq. 5);
                             ignored for Max-Cut                                              */
  float lr, adam_b1, adam_b2, adam_eps; /* Adam hyper-parameters                              */
  void* stream;           /* hipStream_t to enqueue on; NULL = the null stream               */
  gco_alloc_fn dev_alloc; /* may be NULL together with dev_free                              */
  gco_free_fn dev_free;
  void* alloc_user;
} gco_config;

/* Fill *cfg with defaults: MIS, L=2, dim=16, SYM, fp32, per-subgraph weights,
 * trained embeddings, alpha=2, beta=1, lr=1e-2, Adam (0.9, 0.999, 1e-8). */
int gco_default_config(gco_config* cfg);

/* Create / destroy a context bound to the current HIP device.  destroy frees
 * every device buffer the context holds.  EINVAL for an unsupported config. */
int gco_create(const gco_config* cfg, gco_ctx** out);
int gco_destroy(gco_ctx* ctx);

/* The configuration the context was created with. */
int gco_get_config(gco_ctx* ctx, gco_config* out);

/* How the three width-1 passes of the scalar layer (the aggregation before the sigmoid of
 * Eq. 4, the loss of Eq. 5 with its derivative, the first aggregation of back-propagation)
 * are launched.  GCO_SCALAR_AUTO (the default) chooses at gco_upload_graph from the sizes of
 * the subgraphs; the other values force one form (tests, tuning):
 *   STREAMS     three launches, the gathered scalars come from memory (any graph);
 *   STAGED      three launches, each workgroup first copies its subgraph's vector into LDS
 *               (the largest subgraph's float vector must fit a compute unit's LDS twice);
 *   ONE_LAUNCH  one launch with a workgroup per subgraph (two such vectors must fit once).
 * All forms compute the same sums; where a row's entries fall into the 64-entry steps of
 * the kernels differs, so results agree to fp32 rounding, not bit for bit.  Call before
 * gco_upload_graph, which returns GCO_ERANGE if the subgraphs do not fit a forced form.
 * EINVAL for an unknown value. */
enum { GCO_SCALAR_AUTO = 0, GCO_SCALAR_STREAMS = 1, GCO_SCALAR_STAGED = 2, GCO_SCALAR_ONE_LAUNCH = 3 };
int gco_set_scalar_layer_form(gco_ctx* ctx, int form);
/* The form in use for the uploaded graph (one of the three; ESTATE before upload). */
int gco_get_scalar_layer_form(gco_ctx* ctx, int* form);

/* Text of the last failure on ctx (valid until the next call on ctx). */
const char* gco_last_error(gco_ctx* ctx);

/* Upload a graph and its subgraph ids (Alg. 1 inputs "Graph G, subgraph set {G_i}").
 *   n        node count, 1 <= n < 2^31
 *   rowptr   int64[n+1], rowptr[0] = 0
 *   col      int32[rowptr[n]]: symmetric CSR of a simple undirected graph: both
 *            directions present, columns ascending within a row, no self loops,
 *            no duplicates
 *   part_id  int32[n] with values in [0, num_parts), or NULL for one subgraph;
 *            num_parts <= 16384 (ERANGE beyond)
 * Builds on the device: the subgraph-contiguous node order, the CSR of local
 * edges (both ends in one subgraph; only these are trained on, Sec. 3.3), local
 * degrees and the normalisation of Eq. 3, and keeps the full CSR for the
 * cross-edge export.  Resets parameters and optimizer state.
 * EINVAL with a message for a malformed graph; may be called again with a new
 * graph. */
int gco_upload_graph(gco_ctx* ctx, int64_t n, const int64_t* rowptr, const int32_t* col,
                     const int32_t* part_id, int32_t num_parts);

/* Counts: nodes, undirected edges, edges inside subgraphs, edges between them. */
int gco_graph_info(gco_ctx* ctx, int64_t* n, int64_t* m, int64_t* m_local, int64_t* m_cut);

/* Parameters.  E is float[n * dim], row-major, original node order (the random
 * initial embeddings of Sec. 3.2).  W points to num_layers host arrays:
 * W[l-1] is float[Pw * dim * dim] for l < L and float[Pw * dim] for l = L, laid
 * out [subgraph][d_in][d_out] row-major, Pw = num_parts or 1 if weights are
 * shared.  set_params also zeroes the optimizer state and the step counter. */
int gco_set_params(gco_ctx* ctx, const float* E, const float* const* W);
int gco_get_params(gco_ctx* ctx, float* E, float* const* W);

/* The same with the input processing of Sec. 3.2: the initial embeddings pass once through
 * the Gumbel-softmax, which turns every row into a distribution close to a one-hot vector:
 *   X[i, :] = softmax((E[i, :] + g[i, :]) / tau),   g = -log(-log(U)),
 * U is float[n * dim] of uniforms in the open interval (0, 1) supplied by the caller
 * (original node order), tau > 0.  X takes the place of E as the embedding (it is what
 * gco_get_params returns and, if train_embed is set, what is trained); the noise is used
 * this once.  Computed in fp32 on the device.  EINVAL for tau <= 0 or a NULL pointer. */
int gco_set_params_gumbel(gco_ctx* ctx, const float* E, const float* U, float tau,
                          const float* const* W);

/* Adam state, for checkpoints (Alg. 1 stage 1 keeps every subgraph's network and optimizer
 * state): first and second moments shaped like the parameters, and the step counter t.
 * When subgraphs have been trained different numbers of times (gco_train_subset), `step`
 * alone does not describe the state: save gco_get_steps too and restore with
 * gco_set_opt_state followed by gco_set_steps. */
int gco_get_opt_state(gco_ctx* ctx, float* mE, float* vE, float* const* mW, float* const* vW,
                      int64_t* step);
int gco_set_opt_state(gco_ctx* ctx, const float* mE, const float* vE, const float* const* mW,
                      const float* const* vW, int64_t step);

/* Optional per-node term added to the linear coefficient of the objective:
 * L += sum_i extra[i] * p_i (the fine-tuning penalty of Sec. 3.3 is lambda on
 * the listed nodes, 0 elsewhere).  extra = NULL clears it.  float[n]. */
int gco_set_linear_penalty(gco_ctx* ctx, const float* extra);

/* Run `epochs` full-batch training epochs (Sec. 3.2: forward Eq. 3-4, loss
 * Eq. 5, back-propagation, parameter update), all subgraphs at once.  If
 * loss_per_epoch is not NULL it receives double[epochs]: the total loss at the
 * parameters each epoch started from.  Asynchronous when loss_per_epoch is
 * NULL (use gco_sync); otherwise returns after the stream has drained. */
int gco_train(gco_ctx* ctx, int32_t epochs, double* loss_per_epoch);

/* The same for a subset of the subgraphs: the fine-tuning step of Sec. 3.3 / Alg. 1
 * stage 3 retrains only the subgraphs involved in a conflict, warm-started from their
 * current parameters and optimizer state, usually after gco_set_linear_penalty.
 * parts is int32[num_listed] of subgraph ids (host; duplicates allowed).  Subgraphs that
 * are not listed keep their embeddings, weights, Adam moments, step counts and
 * probabilities bit for bit.  With shared weights the one weight set is updated from the
 * gradients of the listed subgraphs only.  loss_per_epoch[e] is the sum of the listed
 * subgraphs' losses.  Every subgraph (and weight set) counts its own Adam steps, so the
 * bias correction of a subgraph depends only on how often that subgraph was trained.
 * ERANGE for an id outside [0, num_parts). */
int gco_train_subset(gco_ctx* ctx, int32_t epochs, const int32_t* parts, int32_t num_listed,
                     double* loss_per_epoch);

/* Adam step counts: steps_embed is int64[num_parts] (embedding rows of each subgraph),
 * steps_weights int64[Pw] (weight sets).  gco_set_params zeroes them; gco_set_opt_state
 * sets all of them to its `step`; gco_get_opt_state reports the largest.  Host arrays. */
int gco_get_steps(gco_ctx* ctx, int64_t* steps_embed, int64_t* steps_weights);
int gco_set_steps(gco_ctx* ctx, const int64_t* steps_embed, const int64_t* steps_weights);

/* Best-by-loss snapshot (Alg. 1 stage 1 stores, per subgraph, the network of the lowest
 * loss).  A model is one subgraph with its embedding rows and its own weight set; with
 * shared weights the whole batch is one model judged by the total loss.  While enabled,
 * every epoch of gco_train / gco_train_subset compares each trained model's loss (the one
 * reported for that epoch, i.e. at the parameters the epoch started from) with the lowest
 * seen so far and, where it is lower, copies those parameters into a device-side
 * snapshot before the update.  enable != 0 starts tracking and forgets earlier snapshots
 * (allocates one more copy of the parameters, fp32); enable == 0 stops tracking and keeps
 * the snapshots.  gco_set_params and a new graph forget them too.  Optimizer state is not
 * part of the snapshot.  With shared weights the one model is judged by the sum over the
 * subgraphs an epoch trains: totals of gco_train and of a gco_train_subset over fewer
 * subgraphs are not comparable, so enable tracking anew before changing the set. */
int gco_keep_best(gco_ctx* ctx, int32_t enable);
/* Lowest loss per model: double[Pw] (host), +infinity for a model never offered. */
int gco_get_best_loss(gco_ctx* ctx, double* best_loss);
/* Copy the snapshots back into the current parameters (models without one keep theirs).
 * Adam moments and step counts are left as they are.  ESTATE if tracking was never on. */
int gco_restore_best(gco_ctx* ctx);

/* Forward pass at the current parameters: the probabilities of Alg. 1 stage 2. */
int gco_forward(gco_ctx* ctx);
/* Probabilities of the last forward / the forward of the last epoch: float[n]. */
int gco_get_probs(gco_ctx* ctx, float* p);
/* Forward + loss at the current parameters: total and, if per_part is not NULL,
 * double[num_parts] per-subgraph values. */
int gco_loss(gco_ctx* ctx, double* total, double* per_part);
/* Test hook for the host side of the work decomposition (no device call): the shares of
 * `target` workgroups that n subgraphs of weight work[k] >= 0 get, share[k] within
 * [lo[k], hi[k]] (0 <= lo[k] <= hi[k]).  The shares add up to exactly `target` whenever
 * sum(lo) <= target <= sum(hi), and to the nearest bound otherwise; units go where the
 * work per unit is largest.  A launch is sized to whole rounds of the workgroups that are
 * resident at once; a handful more would run as a round of their own.
 * All pointers are host memory of n elements.  GCO_EINVAL on null pointers, n < 0,
 * target < 0 or lo[k] > hi[k]. */
int gco_apportion(const double* work, int32_t n, int64_t target, const int32_t* lo, const int32_t* hi,
                  int32_t* share);

/* Forward + backward at the current parameters without an update (test hook):
 * gradients shaped like the parameters. */
int gco_get_grads(gco_ctx* ctx, float* gE, float* const* gW);

/* Hidden activations H_l of the last forward pass, l in [1, num_layers - 1], as
 * float[n * dim] in original node order (test hook; bf16 storage is widened to
 * fp32 exactly).  The ReLU decisions of the backward pass are the signs of
 * these values. */
int gco_get_hidden(gco_ctx* ctx, int32_t layer, float* H);

/* Binarise and repair.  x[i] = (p[i] >= thr) on the fp32 probabilities of the
 * last forward (Sec. 3.3, binarisation at 0.5).  For MIS with repair_scope !=
 * NONE, selected nodes are then visited in the order (p descending, id
 * ascending) and a node is kept iff no neighbour over the scope's edges (LOCAL:
 * inside subgraphs; ALL: every edge) was kept before it.
 *   x                 uint8[n] out
 *   objective         out: |S| for MIS after repair; for Max-Cut the number of
 *                     edges (all edges) whose ends differ
 *   conflicts_before  out: edges (all edges) with both ends selected, before repair
 *   conflicts_after   out: the same after repair           (any of the three may be NULL) */
int gco_round_repair(gco_ctx* ctx, float thr, int32_t repair_scope, uint8_t* x,
                     int64_t* objective, int64_t* conflicts_before, int64_t* conflicts_after);

/* gco_round_repair for callers that cannot allocate device memory (code under HIP graph
 * capture around it, tight serving loops, harnesses that forbid hipMalloc): same arguments,
 * same results bit for bit, but the call's work area (7 bytes per node plus counters) is a
 * fixed block inside the library's code object instead of memory from hipMalloc or the
 * context's allocator hooks; the call allocates and frees nothing.  Limits: n <= 2^21
 * nodes (ERANGE beyond).  Each GPU holds one such block (14.7 MB) for the life of the
 * process, shared by every context on that GPU: calls that overlap in time on one GPU
 * (different streams or threads) race on it and must be serialised by the caller.  The
 * block is looked up on the device that is current at the call, which must be the device
 * the context was created on. */
int gco_round_repair_static(gco_ctx* ctx, float thr, int32_t repair_scope, uint8_t* x,
                            int64_t* objective, int64_t* conflicts_before, int64_t* conflicts_after);

/* Cross edges (Sec. 3.3: edges whose ends lie in different subgraphs), as pairs
 * (u[i], v[i]) with u < v sorted by (u, v).  Two-call pattern: with u = v = NULL
 * only *count is written; otherwise *count is the capacity of u and v on entry
 * (ERANGE if too small) and the number written on return. */
int gco_cut_edges(gco_ctx* ctx, int64_t* count, int32_t* u, int32_t* v);
/* Cross-node mask (Alg. 1 stage 2, "c"): c[i] = 1 iff node i touches a cross edge. uint8[n]. */
int gco_cross_mask(gco_ctx* ctx, uint8_t* c);
/* Conflict edges (Alg. 1 stage 3, first line): the cross edges with x[u] = x[v] = 1,
 * same order and two-call pattern as gco_cut_edges.  x is uint8[n]. */
int gco_conflict_edges(gco_ctx* ctx, const uint8_t* x, int64_t* count, int32_t* u, int32_t* v);

/* Cross-subgraph coordination (Sec. 3.3; Alg. 1 stage 3), for GCO_PROBLEM_MIS: a thin
 * host-side loop over the calls above.  After the subgraphs have been trained, cross edges
 * whose ends are both selected are conflicts; for a conflict (i, j) either i's or j's
 * subgraph is fine-tuned with the penalty lambda on that node (gco_set_linear_penalty +
 * gco_train_subset) so that its probability falls below 0.5.  A tabular Q-learning agent
 * picks the options over `rounds` rounds; the best assignment is returned.
 *
 * The paper leaves the following open; this is the reading implemented (the same, step by
 * step, as the checker's):
 *   score   of an assignment x = [p >= 0.5]: beta |S| - alpha #{edges of the whole graph
 *           inside S} (the negated objective of Eq. 5 at p = x);
 *   base action ("linear cover"): one pass over the current conflict edges in (u, v) order;
 *           an edge with an end already chosen is covered, otherwise the end with the
 *           smaller probability (ties: smaller id) is chosen;
 *   diff    nothing, or the other end at ONE edge where the pass chose (the pass is redone
 *           with that choice forced);
 *   state   x on the ends of the first round's conflict edges; action = the node a diff
 *           brings in (-1: none); unseen Q entries are 0; greedy ties go to the earlier
 *           candidate; round t explores iff uniforms[2t] < epsilon, then takes candidate
 *           floor(uniforms[2t+1] * count);  Q(s,a) += q_lr (r + q_gamma max Q(s',.) - Q(s,a))
 *           with r = the change of the score;
 *   fine-tune: chosen nodes keep the penalty (penalties accumulate); the subgraphs that own
 *           this round's chosen nodes train epochs_per_round epochs;
 *   stop    after `rounds` rounds or when no conflict is left.
 * part_id: int32[n] as given to gco_upload_graph (NULL = one subgraph: nothing to do).
 * uniforms: double[2 * rounds] in [0, 1), supplied by the caller.
 * Outputs (host; each may be NULL except x_best): x_best uint8[n] and *score_best, the
 * assignment of the highest score (the first on ties); actions int32[rounds]; scores
 * double[rounds + 1] and conflicts int64[rounds + 1] (cross conflicts) of every evaluated
 * assignment, entry 0 before the first round; *rounds_run.  The context is left with the
 * penalties and parameters of the last round.  alpha and beta are the context's.  EINVAL
 * for a context that is not GCO_PROBLEM_MIS. */
typedef struct {
  int32_t rounds;
  int32_t epochs_per_round;
  float lambda;            /* penalty coefficient of Sec. 3.3 */
  float q_lr, q_gamma, epsilon;
} gco_rl_config;
int gco_coordinate(gco_ctx* ctx, const int32_t* part_id, const gco_rl_config* rl, const double* uniforms,
                   uint8_t* x_best, double* score_best, int32_t* actions, double* scores,
                   int64_t* conflicts, int32_t* rounds_run);

/* Graph partitioning by modularity (Sec. 3.1): the Louvain heuristic, on the host (no
 * context, no device).  Same graph format as gco_upload_graph (symmetric CSR, no self
 * loops; symmetry is not verified).  Writes part_id[n] (int32, host): community ids
 * 0 .. *num_parts - 1, numbered by smallest member, ready to be passed to
 * gco_upload_graph; *modularity (may be NULL) receives Q of that partition.  Gains are the
 * integers 2 m^2 dQ of Eq. 2, so the result is free of rounding: nodes are visited in
 * ascending id until a sweep moves nothing, a node moves only to a strictly better
 * community (ties: smallest id), communities are merged into nodes level by level, at most
 * max_levels levels.  EINVAL for a malformed graph, ERANGE for 2^31 or more CSR entries. */
int gco_louvain(int64_t n, const int64_t* rowptr, const int32_t* col, int32_t max_levels,
                int32_t* part_id, int32_t* num_parts, double* modularity);

/* Merge the communities of part_id (values in [0, num_parts)) into at most max_parts groups
 * without splitting any, for a bounded number of subgraphs of similar size (merging never
 * cuts an edge; isolated nodes and tiny communities are the usual case).  Communities are
 * taken in the order (size descending, id ascending) and each goes to the group with the
 * fewest nodes so far (ties: smallest group id).  part_out may alias part_id.  Host only.
 * *num_out = min(num_parts, max_parts); with num_parts <= max_parts ids are copied. */
int gco_pack_parts(int64_t n, const int32_t* part_id, int32_t num_parts, int32_t max_parts,
                   int32_t* part_out, int32_t* num_out);

/* Measurement aid (no context): what a plain streaming kernel reaches on the current
 * device, in GB/s of bytes moved, over `repeats` launches on arrays of bytes_per_array
 * bytes (allocated and freed inside; at least 1 MiB).  kind 0: one array read; 1: one array
 * copied to another; 2: three arrays read and written in place (the access pattern of the
 * Adam update of the embeddings).  The benchmark reports the training kernels against
 * these figures beside the published HBM bandwidth. */
int gco_stream_probe(int32_t kind, size_t bytes_per_array, int32_t repeats, double* gbytes_per_s);

/* Wait for the context's stream. */
int gco_sync(gco_ctx* ctx);

/* Per-kernel timing.  With profiling on, every kernel launch of gco_train /
 * gco_forward is bracketed by events on the context's stream (this slows the
 * epoch slightly: an event costs a few microseconds of idle stream).
 * gco_set_profiling(ctx, 2) brackets only the kernel kinds whose bit is set in
 * kind_mask (bit i = kind i); mode 3 brackets every eighth launch of those kinds,
 * counted from this call (the first one included).
 * gco_get_timing: for kernel kind i in [0, gco_num_kernel_kinds()) returns the
 * launches counted and their summed duration in ms since the last reset, and
 * the algorithmic bytes of one launch.  gco_kernel_kind_name gives its name. */
int gco_set_profiling(gco_ctx* ctx, int32_t mode, uint64_t kind_mask);
int gco_num_kernel_kinds(void);
const char* gco_kernel_kind_name(int32_t kind);
int gco_get_timing(gco_ctx* ctx, int32_t kind, int64_t* launches, double* total_ms,
                   double* algorithmic_bytes_per_launch);
int gco_reset_timing(gco_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* GCO_H */
