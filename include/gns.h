/*
 * gns.h -- C ABI of the MI355X (gfx950) Global Neighbor Sampling hot path.
 *
 * Paper: "Global Neighbor Sampling for Mixed CPU-GPU Training on Giant Graphs"
 * (arxiv 2106.06150, KDD'21).  The library implements, on one GPU, the
 * per-mini-batch sampler of Algorithm 1 and the data movement it feeds:
 *
 *   gns_sample_cache     Section 3.2 / Eq. (1) / Theorem 1: the periodic global
 *                        node cache, inclusion driven by node degree
 *   gns_sample_blocks    Algorithm 1 top-down loop; Section 2.1 (uniform
 *                        node-wise sampling), Sections 3.3 and 4.1 (input layer
 *                        restricted to cached neighbors), Section 3.4
 *                        (importance-sampling coefficients); the set union
 *                        B^{l-1} <- B^{l-1} U N_l(u) relabelled into block CSRs
 *   gns_gather_features  Section 2.2 steps 2-3: slice the input-node features
 *                        (cached rows come from the device-resident cache table)
 *   gns_aggregate        Algorithm 1 bottom-up loop, f_l with the mean
 *                        aggregator and Section 3.4's 1/p rescaling
 *
 * General rules
 *  - Every pointer is a DEVICE pointer unless its name starts with host_ or it
 *    is documented as a host pointer (struct pointers, out-parameters).
 *  - The caller owns every buffer, including the workspace; the library
 *    borrows them for the lifetime of the context and never frees them.  All
 *    device memory the kernels touch is the caller's (or, for
 *    gns_sample_blocks_static, the library's fixed scratch array).  What the
 *    library itself allocates is host-side or runtime state: gns_create and
 *    gns_fork allocate a small pinned host mirror of the device counters, HIP
 *    events and a capture stream; the first mini-batch with a new set of block
 *    buffers instantiates a HIP graph of its launch sequence; gns_profile_begin
 *    creates HIP events.  Everything is released by gns_destroy.
 *  - All device work is enqueued on the hipStream_t passed as `hip_stream`
 *    (NULL = the default stream).  Calls that must report counts to the host
 *    (gns_sample_cache, gns_sample_blocks) synchronise that stream before
 *    returning; gns_gather_features and gns_aggregate only enqueue.
 *  - Every call returns a gns_status; nothing aborts or prints.  A message for
 *    the last failure is available from gns_last_error.
 *  - One context serves one stream at a time; calls on the same context must
 *    not overlap.  There is no global state.
 *  - Results are a pure function of (graph, config, seed, epoch, seeds): the
 *    random source is the counter-based Philox4x32-10 generator, so a repeated
 *    call reproduces its output bit for bit.
 *  - Environment variables (testing and tuning aids; none changes a result,
 *    only which kernel or launch shape produces it; the first three are read
 *    when a workspace is sized and when the context is created, and must be
 *    the same at both times):
 *      GNS_MARK_TILE_WORDS=<64..8192, power of two>  words of the frontier
 *        mark bitmap per block of the union step
 *      GNS_MARK_SUMMARY_MIN_WORDS=<n>  bitmaps of at least n words keep a
 *        summary (one bit per word; default 65536)
 *      GNS_COARSE_SHIFT=<1..6>  ids per bit (as a power of two) of the coarse
 *        cache bitmap of graphs whose bitmap does not fit LDS
 *      GNS_NO_COARSE_L2=1  flag pass of such graphs without the coarse bitmap
 *      GNS_FLAG_BLOCKS_PER_CU=<n>  grid of that flag pass (default 2)
 *      GNS_LANE_ROWS_MIN=<n>  UNIFORM layers use the one-row-per-lane sampler
 *        from n rows per launch on (default 262144)
 *      GNS_NO_LANE_SAMPLER=1  never use the one-row-per-lane sampler
 *      GNS_NO_GRAPH=1  enqueue a mini-batch's kernels one by one instead of
 *        replaying a captured HIP graph
 */
#ifndef GNS_H_
#define GNS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define GNS_MAX_LAYERS 8
#define GNS_MAX_FANOUT 64
#define GNS_MAX_GROUP 16     /* mini-batches one gns_*_group call serves */

typedef struct gns_ctx gns_ctx; /* opaque; one per (graph, config, device) */

typedef enum {
    GNS_OK = 0,
    GNS_EINVAL = 1,     /* bad argument (null pointer, size out of range, duplicate or out-of-range seed) */
    GNS_ECAPACITY = 2,  /* a caller buffer or the workspace is too small; nothing was written past it */
    GNS_ESTATE = 3,     /* call order: a cache policy is configured but no cache has been drawn */
    GNS_EHIP = 4,       /* a HIP runtime call failed */
    GNS_ENOMEM = 5,     /* host allocation failed */
    GNS_ENOTIMPL = 6    /* a policy or mode this build does not provide */
} gns_status;

/* Per-layer neighbor-selection policy (Algorithm 1, `sample(N(u), C)`). */
enum {
    GNS_UNIFORM = 0,    /* Section 2.1: min(k, deg(v)) neighbors uniformly without replacement, weight 1 */
    GNS_CACHE_ONLY = 1, /* Sections 3.3 / 4.1: min(k, N_C(v)) of the cached neighbors, weight from Section 3.4 */
    GNS_CACHE_FIRST = 2 /* Section 3.3: as GNS_CACHE_ONLY; a row with fewer than k cached neighbors then draws
                           the shortfall uniformly without replacement from its neighbors outside the cache
                           (slots N_C, N_C + 1, ... of the row's Philox stream); cached neighbors are
                           emitted first; fill weight 1, or |N(v) \ C| / r with GNS_W_UNBIASED */
};

/* Section 3.4 rescaling.  p^C_u = 1 - (1 - deg(u)/nnz)^|C|.
 *  PRINTED:  weight = 1 / (p^C_u * k / min(k, N_C(v)))     (the formula as printed)
 *  UNBIASED: weight = N_C(v) / (min(k, N_C(v)) * p^C_u)    (Horvitz-Thompson form) */
enum { GNS_W_PRINTED = 0, GNS_W_UNBIASED = 1 };

/* The graph G(V, E) of Algorithm 1 as a CSR adjacency, plus the input features.
 * Rows must be sorted ascending and free of duplicates; deg(v) is the row length. */
typedef struct {
    int64_t num_nodes;             /* n = |V|, 1 <= n < 2^31                                   */
    int64_t num_entries;           /* nnz = indptr[n], 1 <= nnz                                */
    const void* indptr;            /* device: int32[n+1] or int64[n+1]                          */
    int32_t indptr_is_i64;         /* 0: int32 offsets, 1: int64 offsets                        */
    const int32_t* indices;        /* device: int32[nnz] neighbor ids                           */
    int32_t feat_dim;              /* F >= 0 (0: no features, gather/cache table unavailable)   */
    const float* feat_dev;         /* device fp32[n x F] row-major, or NULL                     */
    const float* feat_host_pinned; /* pinned host fp32[n x F] readable from the device, or NULL */
} gns_graph;

/* How a CACHE_ONLY layer learns which entries of a dst row point into the cache
 * (Section 3.3).  Both give the identical sample.
 *  GNS_FLAGS_PER_BATCH: every mini-batch streams the CSR segments of its dst rows and
 *      tests each entry against the cache bitmap (the "overlap" computation).
 *  GNS_FLAGS_PER_CACHE: gns_sample_cache tests every CSR entry once and keeps one bit
 *      per entry; mini-batches only read their rows' bits.  This is the induced subgraph
 *      S of Section 3.3 (built once, right after the cache is drawn) in bit form; it
 *      costs num_entries/8 bytes of workspace and one pass over the graph per cache. */
enum { GNS_FLAGS_PER_BATCH = 0, GNS_FLAGS_PER_CACHE = 1 };

/* The probability the cache is drawn with (Section 3.2).
 *  GNS_PROB_DEGREE: Eq. (1), p_i = deg(i) / sum of degrees.
 *  GNS_PROB_WALK:   the random-walk probability P^L = (D_L A + I) ... (D_1 A + I) P^0 of the same
 *      section, P^0 uniform on the training nodes, D_l = diag(min(k_l, deg)/deg) with k_l the
 *      fan-out of the l-th layer counted from the seeds.  gns_cache_walk_probability must run
 *      before gns_sample_cache; the workspace grows by about 24 bytes per node. */
enum { GNS_PROB_DEGREE = 0, GNS_PROB_WALK = 1 };

typedef struct {
    int32_t num_layers;               /* L, 1..GNS_MAX_LAYERS                                       */
    int32_t fanout[GNS_MAX_LAYERS];   /* k per layer; index 0 is layer L (next to the seeds), index
                                         L-1 is layer 1 (the input layer); 1..GNS_MAX_FANOUT        */
    int32_t policy[GNS_MAX_LAYERS];   /* gns_policy per layer, same indexing                          */
    int64_t cache_size;               /* |C|; 0 if no layer uses the cache                          */
    int32_t wmode;                    /* GNS_W_PRINTED / GNS_W_UNBIASED                             */
    int32_t max_seeds;                /* largest mini-batch |B| the context must accept             */
    int32_t flag_mode;                /* GNS_FLAGS_PER_BATCH / GNS_FLAGS_PER_CACHE                  */
    int32_t cache_probability;        /* GNS_PROB_DEGREE (0) / GNS_PROB_WALK                          */
} gns_config;

/* One layer's block: a CSR over (dst rows) x (src columns) in local ids.
 *   src_nodes[0..num_dst)       = the layer's dst nodes in their given order
 *   src_nodes[num_dst..num_src) = the other sampled nodes, ascending global id
 *   indptr[0..num_dst]          = exclusive prefix sum of the per-row counts
 *   indices[e], weights[e]      = local src id and Section 3.4 weight of edge e;
 *                                 a row's edges are in ascending CSR position
 *   row_eligible[r]             = deg(v) (UNIFORM) or N_C(v) (CACHE_ONLY, CACHE_FIRST) of dst row r
 * The five arrays are caller-allocated device buffers with the capacities
 * below (see gns_block_capacity); the three counts are written by the library
 * on the host.  src_nodes of layer l is the dst list of layer l-1.            */
typedef struct {
    int32_t num_dst, num_src, num_edges;
    int32_t* indptr;       /* device int32[cap_dst + 1] */
    int32_t* indices;      /* device int32[cap_edges]   */
    int32_t* src_nodes;    /* device int32[cap_src]     */
    int32_t* row_eligible; /* device int32[cap_dst]     */
    float* weights;        /* device fp32[cap_edges]    */
    int32_t cap_dst, cap_src, cap_edges;
} gns_block;

/* Bytes of device workspace gns_create needs for this graph and config
 * (0 if the arguments are invalid).  Host call, no device work. */
size_t gns_workspace_bytes(const gns_graph* graph, const gns_config* config);

/* Worst-case sizes of block `layer_index` (0 = layer L) for a batch of
 * config->max_seeds seeds: cap_dst = rows, cap_edges = rows * fanout,
 * cap_src = min(rows + edges, n).  gns_sample_blocks requires at least these. */
gns_status gns_block_capacity(const gns_graph* graph, const gns_config* config, int32_t layer_index,
                              int32_t* cap_dst, int32_t* cap_src, int32_t* cap_edges);

/* Creates a context.  `workspace` is a device buffer of at least
 * gns_workspace_bytes bytes, 256-byte aligned, borrowed until gns_destroy.
 * Validates the arguments (GNS_EINVAL), e.g. cache_size must not exceed the
 * number of nodes with at least one neighbor when a cache policy is used.
 * Initialises the workspace on `hip_stream` and synchronises it.
 * A mini-batch's launch sequence is captured into a HIP graph on first use (per set of block buffers)
 * and replayed afterwards, whatever the cache generation;
 * with the environment variable GNS_NO_GRAPH set when the context is created (forks inherit it) every
 * kernel is launched on its own instead. */
gns_status gns_create(gns_ctx** out_ctx, const gns_graph* graph, const gns_config* config,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/* A second context on the same graph, config and cache, for keeping several
 * mini-batches in flight (one context per stream; mini-batches are independent
 * given the cache, as the paper's sampling workers are).  The fork owns its per-batch
 * scratch in `workspace` (gns_fork_workspace_bytes(parent) bytes, 256-byte aligned) and
 * reads the cache structures of the context made by gns_create, which must outlive it.
 * gns_sample_cache is called on that original context only (see there for what may be in
 * flight meanwhile).  Destroy forks with gns_destroy. */
size_t gns_fork_workspace_bytes(const gns_ctx* parent);
gns_status gns_fork(gns_ctx* parent, void* workspace, size_t workspace_bytes, void* hip_stream,
                    gns_ctx** out_child);

gns_status gns_destroy(gns_ctx* ctx);

/* Section 3.2, Eq. (1), Theorem 1.  Draws the cache C for (seed, epoch):
 * the first cache_size distinct nodes of an i.i.d. stream in which node i
 * appears with probability deg(i)/nnz (successive weighted sampling without
 * replacement).  Builds the membership bitmap, the ascending node list, the
 * node -> slot rank index, the per-slot 1/p^C table and, if features were
 * given, the device table of the cached rows' features in slot order.
 * epoch must be < 2^32.  GNS_ECAPACITY if the stream does not yield
 * cache_size distinct nodes within the library's draw limit.  Synchronises hip_stream.
 * The library keeps two copies of these structures: the draw fills the copy that is not in
 * use and makes it the current one when it is complete.  So mini-batches that were enqueued
 * before the call (on this context or on forks, on other streams) may still be in flight:
 * they keep reading the cache they were enqueued with; mini-batches enqueued after the call
 * returns read the new one.  The draw after this one overwrites the copy those older
 * mini-batches read; it waits on the device for them (every draw records an event on each
 * stream each context enqueued mini-batches on since the previous draw, the next draw waits for
 * them), so the host may run ahead freely.  A context may use up to 4 different streams between
 * two draws; gns_sample_blocks(_async) and gns_gather_features return GNS_ESTATE for a fifth.
 * All calls on a context and its forks are made from one host thread at a time. */
gns_status gns_sample_cache(gns_ctx* ctx, uint64_t seed, uint64_t epoch, void* hip_stream);

/* The same draw for callers that prepare the next cache while mini-batches of the current one
 * run (the cache of an epoch depends on (seed, epoch) only).  gns_sample_cache_async enqueues
 * the whole draw into the copy that is not in use and returns without synchronising; it
 * enqueues a fixed number of chunks of the stream (8; a typical cache needs one or two, the
 * rest stand down on the device).  gns_activate_cache makes that copy the current one: from
 * then on gns_sample_blocks / gns_gather_features read it, and the first such call of every
 * context makes its stream wait, on the device, for the draw.  gns_sample_cache is the two
 * calls with a host check in between; after an asynchronous draw that check happens in the
 * next gns_cache_view (GNS_ECAPACITY if the 8 chunks did not yield cache_size distinct nodes:
 * the cache is then incomplete and what was sampled from it is not to be used).
 * GNS_ESTATE if gns_activate_cache finds no draw to make current. */
gns_status gns_sample_cache_async(gns_ctx* ctx, uint64_t seed, uint64_t epoch, void* hip_stream);
gns_status gns_activate_cache(gns_ctx* ctx);

/* Read-only views of the current cache (device pointers into the workspace,
 * valid until the next gns_sample_cache): cache_nodes int32[*cache_size]
 * ascending; bitmap uint64[ceil(n/64)], bit (i & 63) of word (i >> 6) set iff
 * node i is cached; *num_draws = stream draws consumed.  Any out-pointer may
 * be NULL.  GNS_ESTATE before the first draw. */
gns_status gns_cache_view(gns_ctx* ctx, const int32_t** cache_nodes, int64_t* cache_size,
                          const uint64_t** bitmap, int64_t* num_draws);

/* Section 3.2, second approach (config.cache_probability == GNS_PROB_WALK): computes the cache
 * probability from L steps of the recursion above, starting from train_nodes_dev (num_train
 * distinct node ids on the device).  The vector is kept in integers, 2^scale_log2 units per
 * training node (0 <= scale_log2 <= 40), every step rounded down, so the result does not depend on
 * the order of the additions; a draw then picks a uniform integer below the total and takes the
 * node whose prefix interval holds it, and Section 3.4 uses p_u = weight_u / total.
 * GNS_ECAPACITY if a row sum, a product or the total reaches 2^62 (lower scale_log2);
 * GNS_EINVAL for a node id outside [0, n) or an all-zero result.  Synchronises the stream.
 * Call it on the context made by gns_create; it invalidates the current cache: mini-batches
 * already enqueued keep the cache they were enqueued with (the next draw fills the other copy of
 * the cache structures), new ones need a new gns_sample_cache.  No cache draw may be in flight. */
gns_status gns_cache_walk_probability(gns_ctx* ctx, const int32_t* train_nodes_dev, int64_t num_train,
                                      int32_t scale_log2, void* hip_stream);

/* Read-only device views of what gns_cache_walk_probability left: weights uint64[n], their
 * exclusive prefix sum int64[n + 1] (prefix[n] = *total), the number of non-zero weights. */
gns_status gns_cache_probability_view(gns_ctx* ctx, const uint64_t** weights, const int64_t** prefix,
                                      uint64_t* total, int64_t* support);

/* Algorithm 1's top-down loop for one mini-batch.  seeds_dev: num_seeds
 * distinct node ids in [0, n) (1 <= num_seeds <= max_seeds).  `seed` keys the
 * neighbor draws: the draw for (layer l, node v, slot s) uses Philox counter
 * (v, s >> 2, l, 'NBHS') and key (lo32(seed), hi32(seed)), so each row's sample
 * is independent of the batch it appears in.  blocks: host array of
 * num_layers gns_block, index 0 = layer L; their device buffers must have at
 * least the capacities of gns_block_capacity (GNS_ECAPACITY otherwise, before
 * any device work).  On return the counts in every block are valid and the
 * stream has been synchronised.  GNS_EINVAL if a duplicate or out-of-range
 * seed was detected (the blocks' contents are then unspecified). */
gns_status gns_sample_blocks(gns_ctx* ctx, uint64_t seed, const int32_t* seeds_dev, int32_t num_seeds,
                             gns_block* blocks, void* hip_stream);

/* The same work without the final synchronisation, for callers that keep several
 * mini-batches in flight.  gns_sample_blocks_async validates, enqueues the batch's
 * kernels and returns (seeds_dev is read by the first of them: keep it unchanged until
 * the stream has passed that point); until
 * gns_sample_blocks_wait the blocks' host counts hold the placeholder
 * GNS_DEVICE_COUNTS(layer_index), which gns_aggregate understands (see there).
 * gns_sample_blocks_wait copies the counts to the host, synchronises the stream, fills
 * them in and reports GNS_EINVAL if any mini-batch enqueued on the context since the previous
 * wait had a bad seed (not only the last one).  gns_sample_blocks is exactly async followed by wait.
 * Between the two calls no other call may use the context's block state except
 * gns_gather_features / gns_aggregate on the same stream. */
#define GNS_DEVICE_COUNTS(layer_index) (-1 - (layer_index))
gns_status gns_sample_blocks_async(gns_ctx* ctx, uint64_t seed, const int32_t* seeds_dev, int32_t num_seeds,
                                   gns_block* blocks, void* hip_stream);
gns_status gns_sample_blocks_wait(gns_ctx* ctx, gns_block* blocks, void* hip_stream);

/* Several independent mini-batches in one launch sequence.  Mini-batches are independent given the
 * cache (the paper's sampling workers, Section 3.3), and on a GPU the many small dependent kernels
 * of one batch are bound by launch latency, so every kernel of the sequence serves the whole group:
 * batch b of the group runs on context ctxs[b] (count distinct contexts of one family: the context made
 * by gns_create and forks of it, 1 <= count <= GNS_MAX_GROUP), with seed seeds[b], seed nodes
 * seeds_dev[b][0 .. num_seeds[b]) and block buffers blocks[b] (an array of num_layers gns_block each).
 * All arrays are host arrays of count entries.  Results are exactly those of count calls of
 * gns_sample_blocks_async / gns_gather_features / gns_aggregate, one per context, and the same
 * rules hold (placeholders for the counts until the wait, device-side counts with num_nodes[b] < 0
 * or GNS_DEVICE_COUNTS).  Errors are reported on ctxs[0] (gns_last_error(ctxs[0])).
 * The captured launch sequence is kept by ctxs[0] and reused while the group consists of the same
 * contexts and block buffers. */
gns_status gns_sample_blocks_group(gns_ctx* const* ctxs, int32_t count, const uint64_t* seeds,
                                   const int32_t* const* seeds_dev, const int32_t* num_seeds,
                                   gns_block* const* blocks, void* hip_stream);
gns_status gns_sample_blocks_group_wait(gns_ctx* const* ctxs, int32_t count, gns_block* const* blocks,
                                        void* hip_stream);
gns_status gns_gather_features_group(gns_ctx* const* ctxs, int32_t count, const int32_t* const* nodes_dev,
                                     const int32_t* num_nodes, float* const* out_dev, void* hip_stream);
gns_status gns_aggregate_group(gns_ctx* const* ctxs, int32_t count, const gns_block* const* blocks,
                               const float* const* x_src_dev, int32_t feat_dim, float* const* out_dev,
                               void* hip_stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): gns_sample_blocks with the per-batch scratch (device
 * counters, frontier mark bitmap, batch hash map, row extents, sampler scratch, scan partials)
 * in a fixed array of GNS_STATIC_SCRATCH_BYTES bytes that the library holds on every GPU it is
 * loaded on, instead of in the context's workspace.  Same arguments, same results, same errors
 * as gns_sample_blocks; ctx may be the context made by gns_create or any of its forks (the
 * graph, config and current cache are theirs).  The call allocates nothing: no hipMalloc, no
 * host allocation, no HIP graph (the kernels are launched one by one on hip_stream, which is
 * synchronised before the call returns).  GNS_ECAPACITY if the per-batch scratch of this graph
 * and config (what gns_fork_workspace_bytes reports) exceeds the array: nothing is launched.
 * All calls on one GPU share that GPU's array, whatever their context: it is re-initialised at
 * the start of every call, and calls that overlap on one GPU race.  gns_gather_features and
 * gns_aggregate after it take the host counts the call filled in (the device-count
 * placeholders refer to the context's own scratch, which this call does not use). */
#define GNS_STATIC_SCRATCH_BYTES (128u << 20)
gns_status gns_sample_blocks_static(gns_ctx* ctx, uint64_t seed, const int32_t* seeds_dev, int32_t num_seeds,
                                    gns_block* blocks, void* hip_stream);

/* Section 2.2 steps 2-3.  out_dev[j, :] = feature row of nodes_dev[j]
 * (fp32[num_nodes x F] row-major, bit copies).  A cached node is read from the
 * device cache table, any other from feat_dev if given, else from
 * feat_host_pinned.  num_nodes may be 0.  Enqueue only (no synchronisation).
 * num_nodes < 0 means: the number of input nodes (src nodes of the input-layer
 * block) of the last gns_sample_blocks(_async) on this context, read on the device;
 * out_dev must then hold the input layer's cap_src rows. */
gns_status gns_gather_features(gns_ctx* ctx, const int32_t* nodes_dev, int32_t num_nodes, float* out_dev,
                               void* hip_stream);

/* Algorithm 1 bottom-up loop, one layer, mean aggregator with Section 3.4's
 * rescaling: out_dev[v, :] = (1/n_v) * sum over row v's edges of
 * weights[e] * x_src_dev[indices[e], :], n_v = row length, zeros for an empty
 * row.  x_src_dev is fp32[block->num_src x feat_dim], out_dev is
 * fp32[block->num_dst x feat_dim], both row-major.  fp32 arithmetic, edges
 * accumulated in row order.  An edge whose index lies outside [0, num_src) is skipped.  Uses the block's host counts; if block->num_dst is
 * GNS_DEVICE_COUNTS(i) the row count of layer index i is read on the device instead
 * (out_dev must then hold cap_dst rows).  Enqueue only. */
gns_status gns_aggregate(gns_ctx* ctx, const gns_block* block, const float* x_src_dev, int32_t feat_dim,
                         float* out_dev, void* hip_stream);

/* The update step of Algorithm 1 for one layer in its GraphSAGE form (Section 2.1), forward only:
 *   out_dev[r, :] = g( h_self_dev[r, :] . W[0:f1, :] + h_neigh_dev[r, :] . W[f1:f1+f2, :] + bias ),
 * g = max(0, .) if relu != 0, identity otherwise.  h_self_dev is fp32[num_rows x f1] (the dst
 * nodes' own rows: the first num_dst rows of what gns_gather_features wrote), h_neigh_dev
 * fp32[num_rows x f2] (what gns_aggregate wrote), w_dev fp32[(f1 + f2) x hdim] row-major, bias_dev
 * fp32[hdim] or NULL, out_dev fp32[num_rows x hdim]; all row-major device buffers, 16-byte aligned,
 * f1, f2 and hdim multiples of 4 (GNS_EINVAL otherwise).  fp32 matrix-core arithmetic with fp32
 * accumulation; the order of the additions is the kernel's own.  num_rows may be
 * GNS_DEVICE_COUNTS(i): the dst rows of layer index i of the last gns_sample_blocks(_async), read on
 * the device (buffers must then hold that layer's cap_dst rows).  Enqueue only. */
gns_status gns_sage_dense(gns_ctx* ctx, const float* h_self_dev, int32_t f1, const float* h_neigh_dev, int32_t f2,
                          const float* w_dev, const float* bias_dev, int32_t hdim, int32_t relu, float* out_dev,
                          int32_t num_rows, void* hip_stream);

/* Stage timing for benchmarks (no part of the method).  Stages: GNS_STAGE_SAMPLE + i
 * = the sampler launches of layer index i (the first of them also carries the relabel
 * of layer index i - 1); GNS_STAGE_FINISH + i = the union kernels of layer index i (and
 * the last layer's relabel); GNS_STAGE_GATHER; GNS_STAGE_AGGREGATE; GNS_STAGE_PLAN / FLAG /
 * SELECT = the parts of a CACHE_ONLY layer's sampler (also counted in its GNS_STAGE_SAMPLE).
 * gns_profile_begin(ctx, stage_mask, capacity) makes the following calls bracket
 * every launch of a stage whose bit is set in stage_mask with a pair of HIP events on
 * the caller's stream (at most `capacity` pairs are kept, later ones are dropped;
 * stage_mask 0 switches timing off and releases the events).
 * gns_profile_collect(ctx, stage, &total_ms, &launches) synchronises the recorded
 * events of that stage, returns the sum of their elapsed times and their number, and
 * forgets them.  Both are host calls; event creation is the only allocation. */
#define GNS_STAGE_SAMPLE 0
#define GNS_STAGE_FINISH 8
#define GNS_STAGE_GATHER 16
#define GNS_STAGE_AGGREGATE 17
#define GNS_STAGE_PLAN 18   /* CACHE_ONLY, GNS_FLAGS_PER_BATCH: the two work-list kernels          */
#define GNS_STAGE_FLAG 19   /* CACHE_ONLY, GNS_FLAGS_PER_BATCH: the CSR-segment scan (one kernel)  */
#define GNS_STAGE_SELECT 20 /* CACHE_ONLY: the per-row selection kernel                            */
#define GNS_STAGE_DENSE 21  /* gns_sage_dense                                                      */
gns_status gns_profile_begin(gns_ctx* ctx, uint32_t stage_mask, int32_t capacity);
gns_status gns_profile_collect(gns_ctx* ctx, int32_t stage, double* total_ms, int32_t* launches);

/* Message of the last failure on this context (or, for ctx == NULL, of the
 * last failed gns_create / gns_workspace_bytes on this thread).  Never NULL. */
const char* gns_last_error(const gns_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* GNS_H_ */
