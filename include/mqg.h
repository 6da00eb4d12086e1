/*
 * mqg - mini-batch generation for sampled GNN training on one MI355X (gfx950).
 *
 * C ABI of the library.  The four operations are the per-mini-batch data path
 * that the MQ-GNN paper describes around its pipeline: node-wise neighbour
 * sampling, the mini-batch's topology and feature parts, the GPU feature
 * cache with host fallback, and the gather/aggregate (GA) step of GraphSAGE.
 *
 * Conventions
 *   - Every pointer named *_dev / documented "device" must be dereferenceable
 *     by a GPU kernel of the current device (hipMalloc memory, or pinned host
 *     memory from hipHostMalloc where stated).  Pointers documented "host" are
 *     read by the CPU during the call only.
 *   - The caller owns every data buffer (graph, features, cache storage,
 *     block outputs, gathered rows).  A context owns only its private scratch.
 *     The library keeps no caller pointer after a call returns.
 *   - All calls only enqueue work on the given HIP stream and return; results
 *     (including the sizes that depend on the data) are complete when the
 *     stream has been synchronised.  One context serves one stream at a time;
 *     concurrent mini-batches use one context each.
 *   - Every function returns an mqg_status (0 = ok, negative = error).  Errors
 *     that the host can see (null pointers, bad enums, capacities below the
 *     bounds stated below) are returned before anything is enqueued.  No
 *     exception or abort crosses this boundary.
 *   - Blocks are indexed by the GNN layer they feed: block L-1 has the seed
 *     nodes as destinations, block 0 is the outermost and its source nodes
 *     are the rows whose input features are gathered.  fanouts[l] belongs to
 *     block l, so sampling (which walks outward from the seeds) uses
 *     fanouts[L-1] first.
 */
#ifndef MQG_H
#define MQG_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mqg_ctx mqg_ctx;          /* opaque; owns scratch memory only            */
typedef void *mqg_stream;                /* a hipStream_t; NULL is the default stream    */

typedef enum {
    MQG_OK = 0,
    MQG_ERR_INVALID_ARG = -1,            /* null pointer, bad enum, negative size ...    */
    MQG_ERR_CAPACITY = -2,               /* an output buffer is below its stated bound   */
    MQG_ERR_HIP = -3,                    /* a HIP runtime call failed                    */
    MQG_ERR_UNSUPPORTED = -4             /* valid request outside the built limits       */
} mqg_status;

typedef enum { MQG_F32 = 0, MQG_F16 = 1 } mqg_dtype;
typedef enum { MQG_I32 = 0, MQG_I64 = 1 } mqg_itype;

#define MQG_MAX_FANOUT 64                /* per-node neighbour budget of one block       */
#define MQG_MAX_LAYERS 8

/*
 * Graph G = (V, E) in CSR form (paper Sec. III, notation paragraph).  Row v
 * lists the in-neighbours of v (the nodes whose features v aggregates); the
 * cache ranks nodes by this in-degree (Eq. 13).  Preconditions: rows hold no
 * duplicate entry (so distinct adjacency slots are distinct neighbours) and
 * every entry lies in [0, num_nodes); num_nodes < 2^31; every degree < 2^31.
 * Both arrays are device memory and are only read.
 */
typedef struct mqg_graph {
    int64_t num_nodes;
    int64_t num_edges;                   /* length of col_idx                            */
    int32_t ptr_type;                    /* mqg_itype of row_ptr                         */
    int32_t idx_type;                    /* mqg_itype of col_idx and of all node-id I/O  */
    const void *row_ptr;                 /* device [num_nodes + 1]                       */
    const void *col_idx;                 /* device [num_edges]                           */
} mqg_graph;

/*
 * Node feature storage F and the GPU-resident cache C of hot nodes (paper
 * Sec. III "Feature Cache"; Sec. IV "Mini-Batch Transfer To GPU").
 *   feats        the full feature matrix, row v at feats + v*feat_stride
 *                elements.  Pinned host memory (hipHostMalloc) or device
 *                memory; read by GPU kernels directly, so misses travel over
 *                the host link without a staging copy.
 *   cache_rows   device [num_cached x cache_stride]; slot s holds the row of
 *                node cached_ids[s].  NULL together with slot_of == NULL
 *                means "no cache": every row is read from feats (use this
 *                when feats itself is in HBM).
 *   slot_of      device [num_nodes]; cache slot of a node or -1.
 *   cached_ids   device [num_cached], graph idx_type; may be NULL if not wanted.
 * Strides are in elements of dtype.  Rows are moved as opaque bytes.
 */
typedef struct mqg_cache {
    int64_t num_nodes;
    int64_t num_cached;
    int32_t dim;
    int32_t dtype;                       /* mqg_dtype                                    */
    const void *feats;
    int64_t feat_stride;
    void *cache_rows;
    int64_t cache_stride;
    int32_t *slot_of;
    void *cached_ids;
} mqg_cache;

/*
 * One bipartite block (the topology part of a mini-batch, Sec. IV
 * "Mini-Batch Transfer To GPU").  Caller-allocated device buffers:
 *   src_ids  [cap_src]    global ids of the source nodes.  The first num_dst
 *                         entries are the destination nodes, in order, so a
 *                         destination's own previous-layer row (the second
 *                         half of the concatenation in Eq. 16) is row i of the
 *                         source matrix.  The remaining entries are the
 *                         sampled neighbours not among the destinations,
 *                         each once, ascending by id.
 *   indptr   [cap_dst+1]  CSR offsets of the sampled neighbours per destination.
 *   indices  [cap_nnz]    position in src_ids of each sampled neighbour; within
 *                         a row in ascending order of adjacency slot.
 *   sizes    [4]          int64, written on the device: num_dst, num_src, nnz,
 *                         and a flags word (0 = ok; in the innermost block bit 0
 *                         = some seed id was outside [0, num_nodes) and has been
 *                         replaced by node 0, bit 1 = a seed id occurs more
 *                         than once; the batch is then not a valid sample).
 * Capacity bounds checked by mqg_sample_blocks (MQG_ERR_CAPACITY otherwise), with
 * need_dst(L-1) = num_seeds and need_dst(l) = need_src(l+1):
 *   cap_dst >= need_dst,  cap_nnz >= need_nnz = need_dst * fanouts[l],
 *   cap_src >= need_src = max(need_dst, min(num_nodes, need_dst + need_nnz)).
 */
typedef struct mqg_block {
    int64_t cap_dst;
    int64_t cap_src;
    int64_t cap_nnz;
    void *src_ids;
    int32_t *indptr;
    int32_t *indices;
    int64_t *sizes;
} mqg_block;

/* Library version (major*10000 + minor*100 + patch). */
int32_t mqg_version(void);

/*
 * Create a context for graphs of g's size and batches of at most max_seeds
 * seeds expanded with at most max_fanouts[l] (host array, length L) neighbours
 * per node in block l.  Allocates the private scratch on the current HIP
 * device (about 4.2 bytes per graph node plus a few words per sampled edge of
 * the largest batch).  g's array pointers are not read here and may be NULL.
 */
int mqg_ctx_create(mqg_ctx **out, const mqg_graph *g, int32_t max_seeds,
                   const int32_t *max_fanouts, int32_t num_layers);
int mqg_ctx_destroy(mqg_ctx *ctx);

/*
 * Allocate now what a context would otherwise allocate at the first use of an
 * optional path (with a stream synchronisation there), so that the calls
 * themselves only enqueue work.  `what` is a sum of:
 *   MQG_RESERVE_BACKWARD           scratch of the aggregations' backward, for blocks within the
 *                                  context's bounds (about 24 bytes per sampled edge)
 *   MQG_RESERVE_LAYERWISE          scratch of mqg_sample_layerwise and mqg_select_smallest_keys
 *                                  (about 32 bytes per graph node) for up to
 *                                  max(layerwise_rows, max_seeds) rows per block
 *   MQG_RESERVE_DEDUP_HASH         table and sort buffers of MQG_OPT_DEDUP_HASH
 *   MQG_RESERVE_SAMPLING_PRIORITY  tables of mqg_ctx_set_sampling_priority
 *   MQG_RESERVE_CACHE_BUILD        the temporaries of mqg_build_cache(_ex), about 75 bytes per
 *                                  graph node, kept until the context is destroyed.  With them a
 *                                  build allocates and frees nothing, and a build with
 *                                  MQG_CACHE_DEGREE_SAMPLED - the draw the paper repeats every
 *                                  epoch - returns as soon as its kernels are enqueued (builds on
 *                                  one context must then follow one another on one stream).
 *                                  MQG_CACHE_TOP_DEGREE still reads the maximum degree back and
 *                                  the random-walk policies the check of the training ids, so
 *                                  these wait for the stream; the push walk without
 *                                  graph_symmetric still allocates its transposed adjacency.
 * The call itself allocates and may synchronise the device; 0 for `what` does nothing.
 */
typedef enum { MQG_RESERVE_BACKWARD = 1, MQG_RESERVE_LAYERWISE = 2, MQG_RESERVE_DEDUP_HASH = 4,
               MQG_RESERVE_SAMPLING_PRIORITY = 8, MQG_RESERVE_CACHE_BUILD = 16 } mqg_reserve;
int mqg_ctx_reserve(mqg_ctx *ctx, int32_t what, int64_t layerwise_rows);

/* Message of the last failing call on ctx (or of the last failing
 * mqg_ctx_create on this thread when ctx is NULL).  Never NULL. */
const char *mqg_last_error(const mqg_ctx *ctx);

/* Tuning and test switches; see the MQG_OPT_* constants. */
typedef enum {
    MQG_OPT_FORCE_SLOW_SELECT = 1,       /* value != 0: every row with degree > fanout uses the
                                            repeated-minimum selection (test of the rare path) */
    MQG_OPT_PROFILE = 2,                 /* value != 0: bracket every kernel with HIP events
                                            (adds a few microseconds per kernel)              */
    MQG_OPT_MISS_INFLIGHT_BYTES = 3,     /* bytes of host-memory reads the miss gather keeps
                                            outstanding (1 KiB..1 GiB, default 1 MiB): sizes
                                            its grid; enough to saturate the host link without
                                            crowding concurrent streams out of the memory system */
    MQG_OPT_HEAVY_DEGREE = 4,            /* destinations with more neighbours than this (>= 64,
                                            default 2048) are sampled by a whole workgroup
                                            instead of one wavefront; results do not change   */
    MQG_OPT_DEDUP_HASH = 5,              /* value != 0: frontier dedup and relabel through a hash
                                            table and a sort (memory proportional to the
                                            mini-batch) instead of the node-indexed bitmap and
                                            position table (4.2 bytes per graph node); same
                                            blocks, more kernel launches.  The first use
                                            allocates the table (synchronous)                */
    MQG_OPT_LAYERWISE_CANDIDATES = 6     /* how mqg_sample_layerwise finds the candidates of a
                                            layer: 0 = by graph size (default), 1 = a key slot per
                                            node, 2 = a list read off the masses, 3 = a list from
                                            bits set slot by slot; same blocks (test of the paths
                                            that only large graphs take)                      */
} mqg_option;
int mqg_ctx_set_option(mqg_ctx *ctx, int32_t option, int64_t value);

/*
 * With MQG_OPT_PROFILE on: sum of the HIP-event durations (milliseconds) and
 * number of launches of the kernel called `name` since the last reset.  The
 * call synchronises with the recorded events.  Unknown names give 0 launches.
 */
int mqg_ctx_kernel_time(mqg_ctx *ctx, const char *name, double *total_ms, int64_t *launches);
int mqg_ctx_reset_profile(mqg_ctx *ctx);
/* Names of the kernels seen so far, separated by '\n', into buf (host). */
int mqg_ctx_kernel_names(mqg_ctx *ctx, char *buf, int64_t buf_len);

/*
 * Feature cache (paper Sec. III "Feature Cache", Eq. 13: nodes enter the cache
 * by in-degree; here deterministically).  Ranks all nodes by (degree
 * descending, id ascending), assigns cache slot s to the s-th ranked node for
 * s < cache->num_cached, fills slot_of (-1 elsewhere), cached_ids (if not
 * NULL) and copies the cached rows from cache->feats into cache->cache_rows.
 * In: every field of *cache (buffers allocated by the caller).  Temporary
 * device memory (24 bytes per node) is allocated and freed inside the call,
 * which is therefore synchronous with respect to the host - unless
 * mqg_ctx_reserve(MQG_RESERVE_CACHE_BUILD) has set it aside beforehand.
 */
int mqg_build_cache(mqg_ctx *ctx, const mqg_graph *g, mqg_cache *cache, mqg_stream stream);

/*
 * The other ways the paper fills the cache (Sec. III "Feature Cache").
 *   MQG_CACHE_TOP_DEGREE      what mqg_build_cache does.
 *   MQG_CACHE_DEGREE_SAMPLED  Eq. 13 as stated: membership is drawn with probability proportional
 *                             to in-degree, without replacement - a fresh draw for every `seed`
 *                             (the paper rebuilds the cache every epoch).  Every adjacency slot j
 *                             of node v is a ticket with the uniform key
 *                             mix(mix(mix(mix(seed + G) ^ ~0) ^ v) ^ j); a node's key is the minimum
 *                             over its tickets (all ones without neighbours); the num_cached nodes
 *                             with the smallest (key, id) are cached, slot s = s-th smallest.
 *   MQG_CACHE_RANDOM_WALK     Eq. 14-15, for training sets that are a small part of the graph:
 *                             P(0) = 1/num_train on train_ids, 0 elsewhere, then num_steps steps with
 *                             the sampling ratio d_v = min(step_fanouts[l-1], deg_v) / deg_v (0 for an
 *                             empty row), deg_v the length of row v.  With A[v][u] = 1 for u in row(v)
 *                             (row v = the nodes v samples from) and D = diag(d), plan->walk_form
 *                             chooses how Eq. 15's matrix D A + I is applied:
 *                             MQG_WALK_PUSH (0, the default) along the direction in which sampling
 *                               moves, P(l) = (D A + I)^T P(l-1):
 *                                 P(l)[u] = P(l-1)[u] + sum over v with u in row(v) of d_v * P(l-1)[v],
 *                               the terms of u added in ascending order of v.  A node that holds mass
 *                               reaches each node of its row with probability d_v, so P(l)[u] is the
 *                               expected number of times u has entered the sampled frontier: the
 *                               nodes reached from the training set, which is what the cache wants.
 *                               The library transposes the adjacency for this (one stable sort of
 *                               the edges by column: about 24 bytes of temporary device memory per
 *                               edge, fewer than 2^31 edges) unless plan->graph_symmetric is set.
 *                             MQG_WALK_PRINTED (1) Eq. 15 exactly as printed, P a column vector,
 *                               P(l) = (D A + I) P(l-1):
 *                                 P(l)[i] = P(l-1)[i] + d_i * sum_{j in row(i)} P(l-1)[j],
 *                               the row summed in adjacency order, then scaled.  It moves mass
 *                               against the sampling direction; on a directed graph it scores nodes
 *                               that sampling from the training set never reaches, and after one
 *                               step from a uniform start every node of degree >= fanout scores alike.
 *                             On a graph that equals its transpose the push form is
 *                             P(l)[u] = P(l-1)[u] + sum_{v in row(u)} d_v * P(l-1)[v], (A D + I) P.
 *                             plan->graph_symmetric != 0 states that the graph equals its transpose
 *                             and that every row is in ascending order of id; the push form then sums
 *                             over the adjacency rows themselves and builds nothing.  The statement is
 *                             not checked: if it is false the result is that row-wise sum, not the
 *                             push form (no access leaves the arrays either way).
 *                             Double precision, products rounded on their own.  The num_cached nodes
 *                             of highest P(num_steps) are cached (ties: lower id).  scores_out
 *                             (device double [num_nodes], may be NULL) receives P(num_steps).
 *                             Membership is the deterministic top of the score, not a draw from it.
 *                             A training id outside [0, num_nodes) is never used as an index: it is
 *                             skipped and the call returns MQG_ERR_INVALID_ARG once the work is done.
 *   MQG_CACHE_RANDOM_WALK_SAMPLED  the same scores, membership drawn from them (the text after
 *                             Eq. 15 takes P(L) as the probability of entering the cache): weighted
 *                             sampling without replacement by an exponential race, key_i =
 *                             ticket_i / P(num_steps)[i] in double (+inf for a zero score),
 *                             ticket_i = -log2(r_i / 2^64) in fixed point with 32 fractional
 *                             bits, computed in integers by 32 squarings of the 64-bit mantissa
 *                             (truncated products), r_i = mix(mix(mix(mix(seed + G) ^ ~1) ^ i));
 *                             the num_cached smallest (key, id) are cached, slot s = s-th
 *                             smallest.
 * train_ids: device [num_train], graph idx_type, ids in [0, num_nodes); step_fanouts: host.
 */
typedef enum { MQG_CACHE_TOP_DEGREE = 0, MQG_CACHE_DEGREE_SAMPLED = 1, MQG_CACHE_RANDOM_WALK = 2,
               MQG_CACHE_RANDOM_WALK_SAMPLED = 3 } mqg_cache_policy;

typedef enum { MQG_WALK_PUSH = 0, MQG_WALK_PRINTED = 1 } mqg_walk_form;

typedef struct mqg_cache_plan {
    int32_t policy;                      /* mqg_cache_policy                             */
    int32_t num_steps;                   /* RANDOM_WALK: number of steps L, 0..MQG_MAX_LAYERS */
    uint64_t seed;                       /* DEGREE_SAMPLED, RANDOM_WALK_SAMPLED          */
    const void *train_ids;               /* RANDOM_WALK                                  */
    int64_t num_train;
    const int32_t *step_fanouts;         /* RANDOM_WALK: host [num_steps], each >= 1     */
    double *scores_out;                  /* RANDOM_WALK: optional                        */
    int32_t walk_form;                   /* RANDOM_WALK: mqg_walk_form                   */
    int32_t graph_symmetric;             /* RANDOM_WALK, push form: see above            */
} mqg_cache_plan;

/* mqg_build_cache with a choice of policy; plan == NULL means MQG_CACHE_TOP_DEGREE.  Otherwise as
 * mqg_build_cache (buffers in *cache, temporary device memory, synchronous with the host). */
int mqg_build_cache_ex(mqg_ctx *ctx, const mqg_graph *g, mqg_cache *cache, const mqg_cache_plan *plan,
                       mqg_stream stream);

/*
 * L-hop fixed-fanout node-wise neighbour sampling into blocks (paper Sec.
 * III-A, GraphSAGE paragraph: a fixed number of neighbours of every node of a
 * layer, drawn uniformly at random, a fresh draw per layer).
 *   seeds_dev  device [num_seeds], graph idx_type, distinct, in [0, num_nodes)
 *              (violations are flagged in blocks[L-1].sizes[3]; an id out of range
 *              is never used as an index)
 *   fanouts    host [num_layers], 1..MQG_MAX_FANOUT, indexed by block
 *   blocks     host array of num_layers descriptors (see mqg_block)
 * For each destination v of block l with adjacency row of length d: all d
 * neighbours if d <= fanouts[l]; otherwise the fanouts[l] adjacency slots j
 * with the smallest (key, j), key = mix(mix(mix(mix(rng_seed + G) ^ l) ^ v) ^ j)
 * with mix the SplitMix64 finaliser and G = 0x9E3779B97F4A7C15 - sampling
 * without replacement, a pure function of (rng_seed, l, v, j).
 */
int mqg_sample_blocks(mqg_ctx *ctx, const mqg_graph *g, const void *seeds_dev, int32_t num_seeds,
                      const int32_t *fanouts, int32_t num_layers, uint64_t rng_seed,
                      mqg_block *blocks, mqg_stream stream);

/*
 * mqg_sample_blocks with the sampling seed read from device memory when the
 * kernels run, for callers that record a mini-batch step into a HIP graph and
 * replay it: a recorded launch keeps its arguments, so what changes from one
 * replay to the next - the seeds in seeds_dev[0..num_seeds) and *rng_seed_dev -
 * has to live in buffers that the caller rewrites between replays.  Same
 * blocks as mqg_sample_blocks(..., rng_seed = *rng_seed_dev, ...).  With the
 * default dedup path and MQG_OPT_PROFILE off, this call, mqg_gather_features
 * and mqg_sage_mean_aggregate only enqueue kernels (no allocation, no memset,
 * no synchronisation) and can be captured.
 */
int mqg_sample_blocks_seed_dev(mqg_ctx *ctx, const mqg_graph *g, const void *seeds_dev, int32_t num_seeds,
                               const int32_t *fanouts, int32_t num_layers,
                               const uint64_t *rng_seed_dev, mqg_block *blocks, mqg_stream stream);

/*
 * Layer-wise sampling after LADIES (paper Sec. III-B, Eq. 6-9) into blocks of
 * the same layout, with edge weights.  blocks[L-1] has the seeds as rows; for
 * every block, from L-1 down to 0, with rows D:
 *   - column masses in integers: mass_i = sum over v in D with i in N(v) or
 *     i == v of floor(2^40 / (deg_v + 1)); q_i = mass_i / (deg_i + 1) is 2^40
 *     times the squared column norm ||R P_{*,i}||^2 of Eq. 7, P = D^-1/2 (A + I)
 *     D^-1/2 (Eq. 2); the candidates (Eq. 6) are the nodes with mass_i > 0;
 *   - layer_sizes[l] candidates are drawn without replacement with probability
 *     proportional to q_i (all of them if there are no more), by an
 *     exponential race: key_i = ticket_i * (deg_i + 1) / mass_i in doubles,
 *     ticket_i as for MQG_CACHE_RANDOM_WALK_SAMPLED from r_i =
 *     mix(mix(mix(mix(rng_seed + G) ^ (64 + l)) ^ i)); the smallest (key, id) win;
 *   - src_ids = the drawn nodes, ascending (they are the rows of block l-1;
 *     unlike mqg_sample_blocks the rows are not repeated among the sources);
 *     row v lists the drawn nodes among v itself and its adjacency row, the
 *     self edge first, then in slot order; edge_w[l][p] = P_vi / (s p_i) (Eq. 8),
 *     s the number of drawn nodes and p_i = q_i / sum_j q_j, divided by the
 *     row's sum if normalise != 0 (the normalisation of the sampled operator
 *     the paper mentions after Eq. 9; rows without an edge stay empty).
 * Which nodes are drawn is a pure function of the arguments (integer masses,
 * correctly rounded double operations); the weights are computed in double and
 * rounded to float.
 *   seeds_dev    device [num_seeds], graph idx_type, distinct; an id outside
 *                the graph is replaced by node 0 and flagged (sizes[3] bit 0)
 *   layer_sizes  host [num_layers], each >= 1
 *   blocks       host [num_layers]; block l needs cap_dst >= its number of rows
 *                (num_seeds for L-1, else min(N, layer_sizes[l+1])), cap_src >=
 *                min(N, layer_sizes[l]); edges beyond cap_nnz are dropped and
 *                flagged (sizes[3] bit 2; sizes[2] is then cap_nnz)
 *   edge_w       host array of num_layers device pointers, [cap_nnz] floats each
 * method MQG_LAYERWISE_FASTGCN (paper Sec. III-B, FastGCN paragraph, Eq. 4): the
 * masses are taken over all rows of the graph instead of the block's rows - the
 * squared column norms of P itself, computed at the first such call on the
 * context - so every node is a candidate and the draw does not depend on the
 * mini-batch; everything else is the same (drawn without replacement,
 * importance weights P_vu / (s p_u)).
 * method | MQG_LAYERWISE_DEBIAS (the "+debias" variants, paper Eq. 12): a drawn
 * node's column is scaled by its debiased coefficient beta instead of 1 / (s p),
 * edge_w = P_vi * beta_i (then the row normalisation, if asked for).  With the
 * drawn nodes in the order of the race (ascending (key, id)), n candidates,
 * a_r = n / ((n - r)(r + 1)) for the r-th draw (r from 0) and p_r = q_r / sum_j
 * q_j: the coefficient of a node is a_r (1 - p_0 - ... - p_{r-1}) / p_r when it
 * is drawn and becomes (1 - a_u) beta + a_u at every later draw u; when every
 * candidate is drawn, beta = 1.  Computed in double.
 * method | MQG_LAYERWISE_FLAT (the "+flat" variants, paper Eq. 10): nodes are
 * drawn with probability proportional to sqrt(q_i), the column norm itself
 * instead of its square - the distribution that minimises the variance of the
 * sampled product P (H W) when the rows of H W have equal norms, which is the
 * assumption the paper states (the printed right-hand side names the unknown
 * H W).  key_i = ((ticket_i * ticket_i) * (deg_i + 1)) / mass_i, the order of
 * ticket_i / sqrt(q_i); p_i = sqrt(q_i) / sum_j sqrt(q_j) in the weights and in
 * the debiased coefficients.  The three flags combine freely.
 * The first call allocates context scratch of about 32 bytes per graph node
 * (8 more for FastGCN) and synchronises the stream once.  Feed the blocks to
 * mqg_weighted_aggregate with self_w == NULL.
 */
typedef enum { MQG_LAYERWISE_LADIES = 0, MQG_LAYERWISE_FASTGCN = 1, MQG_LAYERWISE_DEBIAS = 2,
               MQG_LAYERWISE_FLAT = 4 } mqg_layerwise_method;

int mqg_sample_layerwise(mqg_ctx *ctx, const mqg_graph *g, const void *seeds_dev, int32_t num_seeds,
                         const int32_t *layer_sizes, int32_t num_layers, uint64_t rng_seed,
                         int32_t normalise, int32_t method, mqg_block *blocks,
                         float *const *edge_w, mqg_stream stream);

/*
 * The selection step of mqg_sample_layerwise on its own (the k smallest race
 * keys win the draw of Eq. 6-9): bit c of out_bitmap is set iff key c is among
 * the k smallest (key, index) pairs of keys[0..n) - all of them if n <= k; keys
 * that are exactly equal are taken in ascending index order.  A radix select:
 * two counting passes over the 25 leading bits, then the keys that share the
 * threshold's leading bits are settled as a short list.
 *   keys_dev        device [n] unsigned 64-bit keys
 *   out_bitmap_dev  device [ceil(n / 32)] words, written by the call
 * Uses the layer-wise sampler's context scratch (allocated at the first use; with
 * more keys than the graph has nodes, 12 more bytes per key, allocated and kept
 * at the first such call, after a stream synchronisation).
 */
int mqg_select_smallest_keys(mqg_ctx *ctx, const uint64_t *keys_dev, int64_t n, int64_t k,
                             uint32_t *out_bitmap_dev, mqg_stream stream);

/*
 * The selection step of mqg_sample_blocks for one row on its own (paper
 * Sec. III-A: s_node neighbours of a node drawn uniformly, here the k smallest
 * random keys): among `count` candidates, each a (key, slot word) pair, the k
 * first in the order (bit 31 of the slot word if `prioritised`, key, low 31
 * bits of the slot word) are chosen - the binary radix select on wavefront
 * ballots that the sampling kernels run after their threshold pass, exposed
 * so that a test can feed it keys with ties.
 *   keys_dev, slot_words_dev  device [count], 1 <= k <= count <= 256
 *   ordered         non-zero: the candidates are stored in ascending slot
 *                   order (as the one-wavefront-per-row path stores them), so
 *                   equal keys are resolved by position; zero: by slot value
 *                   (the hub path, whose candidates arrive in any order)
 *   out_mask_dev    device [8] words: bit c of the 256-bit mask = candidate c chosen
 */
int mqg_select_row_candidates(mqg_ctx *ctx, const uint64_t *keys_dev, const uint32_t *slot_words_dev,
                              int32_t count, int32_t k, int32_t prioritised, int32_t ordered,
                              uint32_t *out_mask_dev, mqg_stream stream);

/*
 * The ticket of the exponential races on its own (the draw from the random-walk
 * scores after Eq. 15 and the layer-wise draws of Eq. 6-10 race with key =
 * ticket / weight): tickets_dev[i] = ticket(r_i), r_i = mix(mix(mix(mix(seed + G)
 * ^ tag) ^ (first + i))) - slot 0 of node first + i in the key domain `tag` -
 * and ticket(r) = -log2(r / 2^64) in fixed point with 32 fractional bits as
 * described for MQG_CACHE_RANDOM_WALK_SAMPLED.  A pure integer function, exposed
 * so that a test can compare a long stretch of the stream, over thousands of
 * workgroups, with the same function computed on the CPU.
 *   tickets_dev  device [n] unsigned 64-bit
 */
int mqg_exp_tickets(mqg_ctx *ctx, uint64_t seed, int64_t tag, int64_t first, int64_t n,
                    uint64_t *tickets_dev, mqg_stream stream);

/*
 * Cache-prioritised neighbour sampling (paper Sec. I on global neighbour
 * sampling: the sampler prefers neighbours that are in the cache, which cuts
 * the number of distinct uncached rows a mini-batch needs).  After this call
 * every mqg_sample_blocks on `ctx` chooses, for a row with more neighbours than
 * the fanout k, the first k slots in the order (not cached, key, slot) with the
 * keys of mqg_sample_blocks: with c cached neighbours the row keeps min(k, c)
 * of them, uniformly, and fills up with uncached ones, uniformly.  Rows of at
 * most k neighbours are kept whole as before.
 * cache: membership is read from cache->slot_of (device, >= 0 = cached) into a
 * bitmap of num_nodes bits, and the number of cached neighbours of every node
 * of `graph` is tabulated (one pass over the adjacency, 4 bytes per node), both
 * owned by the context, on `stream`; call again after the cache has been
 * rebuilt.  cache == NULL switches back to the uniform draw (graph is then not
 * read).  The first call allocates the two tables.
 */
int mqg_ctx_set_sampling_priority(mqg_ctx *ctx, const mqg_graph *graph, const mqg_cache *cache,
                                  mqg_stream stream);

/*
 * Feature gather through the cache (paper Sec. IV "Mini-Batch Transfer To
 * GPU": rows of cached nodes come from GPU memory, the others from host
 * memory).  out[i, 0:dim] = F[ids[i], 0:dim] byte for byte.
 *   ids_dev      device [cap_ids], graph idx_type (normally blocks[0].src_ids)
 *   num_ids_dev  device int64: number of valid ids (normally &blocks[0].sizes[1]);
 *                values above cap_ids are clamped to cap_ids
 *   out_dev      device [cap_ids x out_stride] elements of cache->dtype; in a written row
 *                the elements from dim up to out_stride (padding) are unspecified: when
 *                source and destination rows are 64-byte (16-byte) aligned and long enough
 *                the copy is rounded up to whole 64-byte lines (16-byte words)
 *   stats_dev    device int64[2]: rows served from the cache, rows served
 *                from feats; may be NULL
 * An id outside [0, cache->num_nodes) is never used as an index: its output row
 * is left untouched and it counts in neither stat, so stats[0] + stats[1] below
 * the number of ids tells the caller that some were invalid.
 */
int mqg_gather_features(mqg_ctx *ctx, const mqg_cache *cache, int32_t idx_type,
                        const void *ids_dev, const int64_t *num_ids_dev, int64_t cap_ids,
                        void *out_dev, int64_t out_stride, int64_t *stats_dev, mqg_stream stream);

/*
 * The two halves of mqg_gather_features as calls of their own, for a pipeline
 * that keeps the host link busy (paper Sec. IV: transfer of one mini-batch
 * overlaps sampling and computation of others): the rows that come over the
 * host link are then copied on a stream that does nothing else, one
 * mini-batch after the other, while ids are classified and cached rows copied
 * elsewhere.
 *   mqg_gather_features_cached  looks the ids up, copies the rows found in the
 *       cache (HBM to HBM), writes both counts to stats_dev, and leaves the list
 *       of the other rows in the context;
 *   mqg_gather_features_missed  copies those rows from cache->feats.
 * Same arguments as mqg_gather_features; the pair, in this order, gives the
 * same rows and stats.  Every _cached call on a context must be followed by its
 * _missed call (same arguments) before the context gathers again, and the
 * caller orders the two (same stream, or an event) - the second reads what the
 * first left.  Without a cache (slot_of == NULL) every row belongs to the
 * second call and the first does nothing.
 */
int mqg_gather_features_cached(mqg_ctx *ctx, const mqg_cache *cache, int32_t idx_type,
                               const void *ids_dev, const int64_t *num_ids_dev, int64_t cap_ids,
                               void *out_dev, int64_t out_stride, int64_t *stats_dev, mqg_stream stream);
int mqg_gather_features_missed(mqg_ctx *ctx, const mqg_cache *cache, int32_t idx_type,
                               const void *ids_dev, const int64_t *num_ids_dev, int64_t cap_ids,
                               void *out_dev, int64_t out_stride, int64_t *stats_dev, mqg_stream stream);

/*
 * mqg_gather_features for callers that cannot allocate device memory: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  It
 * takes no context (creating one allocates): the hit and miss lists and the
 * counters that mqg_gather_features keeps in its context live in a device array
 * of fixed size inside the library, MQG_GATHER_STATIC_MAX_IDS entries per list
 * (16 MiB + 64 bytes in all, held by every GPU the library runs on until the
 * process ends).  No call to hipMalloc, hipFree or any allocating routine is
 * made, at the first call or later; the first call on a device only looks up
 * the array's address there.  Same arguments, kernels, results and stats as
 * mqg_gather_features.  With a cache (slot_of != NULL) cap_ids above
 * MQG_GATHER_STATIC_MAX_IDS is refused with MQG_ERR_CAPACITY before anything
 * is enqueued; without a cache there is no limit (no list is used).  The
 * message of a failing call is read with mqg_last_error(NULL).  All calls on a
 * GPU share that GPU's array: two calls whose kernels can overlap there (two
 * streams, two threads) race, so keep them on one stream or order them with
 * events.
 */
#define MQG_GATHER_STATIC_MAX_IDS 1048576
int mqg_gather_features_static(const mqg_cache *cache, int32_t idx_type, const void *ids_dev,
                               const int64_t *num_ids_dev, int64_t cap_ids, void *out_dev,
                               int64_t out_stride, int64_t *stats_dev, mqg_stream stream);

/*
 * GraphSAGE mean aggregation over one block (paper Eq. 16,
 * Z_agg(v) = Mean(H(v)); the GA step "AH" of Sec. IV "Computation").
 *   out[i, c] = (1/n_i) * sum_{e in row i} x_src[indices[e], c],  n_i = row length;
 *   a destination with no sampled neighbour gets zeros.
 * x_src: device [num_src x x_stride]; out: device [cap_dst x out_stride];
 * strides in elements (columns from dim up to out_stride of a written row are
 * unspecified: with 16-byte aligned rows on both sides whole 16-byte words are
 * processed); sums are accumulated in fp32 in row order; MQG_F16
 * rounds once, to nearest even, at the store.
 */
int mqg_sage_mean_aggregate(mqg_ctx *ctx, const mqg_block *block, const void *x_src,
                            int64_t x_stride, void *out, int64_t out_stride, int32_t dim,
                            int32_t dtype, mqg_stream stream);

/*
 * Backward of the mean aggregation (paper Sec. IV "Computation": the gradient
 * of the GA step is the transposed product "AG", G the gradient matrix).  With
 * out = M x_src the forward operator of the block, M[i, s] = 1/n_i for every
 * edge of destination i that points to source s, this computes
 *   grad_x[s, c] = sum over edges (i -> s) of grad_out[i, c] / n_i
 * for all num_src sources (zeros where no edge points).
 * grad_out: device [num_dst x go_stride]; grad_x: device [cap_src x gx_stride];
 * strides in elements, padding columns of written rows unspecified as in the
 * forward.  The edges are first ordered by source with a stable radix sort and
 * each source's terms are added in ascending destination order in fp32, so
 * the result is reproducible bit for bit.  The first call (and any call with
 * larger block capacities than seen before) allocates context scratch of
 * about 20 bytes per edge and synchronises the stream once to do so.
 */
int mqg_sage_mean_aggregate_backward(mqg_ctx *ctx, const mqg_block *block, const void *grad_out,
                                     int64_t go_stride, void *grad_x, int64_t gx_stride, int32_t dim,
                                     int32_t dtype, mqg_stream stream);

/*
 * Weights of the sampled estimator of the graph convolution P H (paper Eq. 1-3),
 * P = D^-1/2 (A + I) D^-1/2 with D_ii = deg(v_i) + 1 (Eq. 2).  For block edge p
 * from destination i (node v_i) to source indices[p] (node v_j)
 *   edge_w[p] = deg(v_i) / n_i * 1 / sqrt((deg(v_i) + 1) (deg(v_j) + 1)),
 * n_i = the number of neighbours the block holds for v_i (Eq. 3 with s_node
 * read as the number actually drawn: a row kept whole has factor 1), and
 *   self_w[i] = P_ii = 1 / (deg(v_i) + 1)
 * is the diagonal term of A + I, which is never part of the sampled set.
 * deg is the length of the node's adjacency row in `graph`.  block->src_ids
 * must hold the sources' global ids, as mqg_sample_blocks writes them.
 * edge_w: device [cap_nnz] floats, self_w: device [cap_dst] floats; entries
 * 0..nnz-1 and 0..num_dst-1 are written (computed in double precision, rounded
 * once).  Enqueued on `stream`; nothing is allocated.
 */
int mqg_gcn_edge_weights(mqg_ctx *ctx, const mqg_graph *graph, const mqg_block *block,
                         float *edge_w, float *self_w, mqg_stream stream);

/*
 * Weighted aggregation over one block (the estimator of paper Eq. 1-3 with the
 * weights above, or any other per-edge weights, e.g. those of a layer-wise
 * sampler, Eq. 4-9):
 *   out[i, c] = self_w[i] * x_src[i, c] + sum over edges p of row i of
 *               edge_w[p] * x_src[indices[p], c]
 * self_w may be NULL (no diagonal term).  Layout, strides, dtype, padding and
 * accumulation as mqg_sage_mean_aggregate (fp32 sums in row order, the
 * diagonal term first).
 */
int mqg_weighted_aggregate(mqg_ctx *ctx, const mqg_block *block, const float *edge_w,
                           const float *self_w, const void *x_src, int64_t x_stride, void *out,
                           int64_t out_stride, int32_t dim, int32_t dtype, mqg_stream stream);

/*
 * Its backward (the transposed product, paper Sec. IV "Computation"):
 *   grad_x[s, c] = sum over edges p = (i -> s) of edge_w[p] * grad_out[i, c]
 *                  (+ self_w[s] * grad_out[s, c] for s < num_dst)
 * Buffers, ordering, reproducibility and scratch as
 * mqg_sage_mean_aggregate_backward (24 bytes of scratch per edge).
 */
int mqg_weighted_aggregate_backward(mqg_ctx *ctx, const mqg_block *block, const float *edge_w,
                                    const float *self_w, const void *grad_out, int64_t go_stride,
                                    void *grad_x, int64_t gx_stride, int32_t dim, int32_t dtype,
                                    mqg_stream stream);

/*
 * Depth of the mini-batch queue, i.e. how many mini-batches to keep in flight
 * (paper Sec. IV "Determining Optimal Queue Size", Eq. 22 and 23):
 *   C = floor(M_Q / M_batch),  M_Q = total_mem - peak_mem * (1 + margin_percent/100)
 *   Q = min(C, max(2, ceil(max_prepare_ms / mean_compute_ms)))
 * max_prepare_ms is the largest observed sampling + transfer time of a
 * mini-batch, mean_compute_ms the mean time of the stage that consumes it,
 * peak_mem the measured peak device memory of one training epoch, margin the
 * paper's 5-10 % safety margin, mem_per_batch the device memory one queued
 * mini-batch holds.  Host arithmetic only (doubles for the times, integers
 * for the memory); no GPU is touched.  The rule presumes a pipeline that waits
 * for its consumer: where preparation is bound by something a deeper queue
 * cannot hide (here: the host link), the depth it gives is harmless but buys
 * nothing beyond the first few.  *cap_out (may be NULL) receives C,
 * *queue_size_out receives Q.  MQG_ERR_INVALID_ARG for non-positive times or
 * sizes, a margin outside 0..100, or peak memory above the total.
 */
int mqg_queue_size(double max_prepare_ms, double mean_compute_ms, int64_t total_mem_bytes,
                   int64_t peak_mem_bytes, int32_t margin_percent, int64_t mem_per_batch_bytes,
                   int64_t *cap_out, int64_t *queue_size_out);

#ifdef __cplusplus
}
#endif
#endif /* MQG_H */
