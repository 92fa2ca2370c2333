/*
 * commrand.h -- C ABI of libcommrand.so: the single-GPU hot path of COMM-RAND
 * mini-batch GNN training (community-structure-aware randomized mini-batching)
 * as hand-written HIP kernels for gfx950 (MI355X).
 *
 * The calls follow Algorithm 1 of the paper (mini-batch training of an L-layer
 * GNN): Step-1 root node partitioning (cr_build_batches), Step-2 sub-graph
 * construction (cr_sample_blocks), then training on the sub-graph
 * (cr_gather_aggregate_*, cr_sage_linear_*, cr_softmax_xent).  Further down:
 * the validation pass (cr_count_correct), GCN on the same blocks (cr_gcn_*) and
 * the software-managed feature cache of the paper's sensitivity study
 * (cr_cache_*, cr_stage_rows, cr_host_alloc).
 *
 * Conventions
 *  - Every function returns a cr_status; cr_last_error() gives the text of the
 *    calling thread's last failure.  No exception crosses this boundary.
 *  - "device" pointers are HIP device memory on the current device; "host"
 *    pointers are ordinary memory.  The library never allocates or frees device
 *    memory: graph, table, outputs and workspaces are caller-owned and only
 *    borrowed for the duration of the enqueued work.  (The one allocation the
 *    library makes, on request, is pinned host memory: cr_host_alloc.)
 *  - All work is enqueued on the given hipStream_t (passed as void*, NULL = the
 *    default stream) and the call returns without synchronising, except where
 *    stated.  Arguments are validated on the host before anything is launched;
 *    under a context created with CR_CTX_DRY_RUN calls stop after validation (no GPU needed).
 *  - Device pointers must be 16-byte aligned.  Row strides (ld*) are in
 *    elements and must make every row 16-byte aligned.
 *  - Sizes that depend on the sampled data (rows, edges, frontier length of a
 *    block) live in a small device-resident header per block; kernels read them
 *    there, so no host round trip is needed between the calls of one batch.
 *  - bf16 values are raw uint16_t bit patterns (upper half of an IEEE float32).
 */
#ifndef COMMRAND_H
#define COMMRAND_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t cr_status;
enum {
    CR_OK = 0,
    CR_ERR_INVALID_ARG = 1, /* null / misaligned pointer, knob out of range, shape mismatch */
    CR_ERR_CAPACITY = 2,    /* a caller-provided buffer or workspace is too small */
    CR_ERR_UNSUPPORTED = 3, /* valid request outside what the kernels were built for */
    CR_ERR_HIP = 4,         /* the HIP runtime reported an error */
    CR_ERR_ASYNC_OVERFLOW = 5 /* cr_ctx_poll_error only: a kernel found a data-dependent size beyond the caller's capacity */
};

#define CR_MAX_LAYERS 8
#define CR_MAX_FANOUT 64
#define CR_HDR_WORDS 8 /* int32 words per block header */
/* header word indices */
#define CR_HDR_N_DST 0
#define CR_HDR_N_SRC 1
#define CR_HDR_NNZ 2
#define CR_HDR_STATUS 3 /* 0 = valid; otherwise CR_ASYNC_* bits: the block did not fit its arrays and must not be used
                           (never with the capacities of cr_block_capacities) */

const char *cr_last_error(void);
const char *cr_version(void);

/* ------------------------------------------------------------------------- */
/* Contexts.  Algorithm 1's loop runs one mini-batch after the other without   */
/* the host looking at any sampled size, so a size that exceeds a caller's     */
/* capacity can only be reported after the fact: kernels record it in device   */
/* status words, and the caller polls them when it chooses (once per epoch,    */
/* say).  A context carries those words and the dry-run flag.  It is a small   */
/* host object; the entry points below take no context argument: they follow   */
/* the context that is CURRENT on the calling thread (none by default).        */
/* ------------------------------------------------------------------------- */
typedef struct cr_ctx cr_ctx;
#define CR_CTX_DRY_RUN 1u       /* calls made under this context validate their arguments on the host and return
                                   without touching the GPU (error paths can be exercised without a device) */
#define CR_CTX_STATUS_WORDS 2   /* status[0]: OR of CR_ASYNC_* bits, sticky; status[1]: the largest size that was needed */
#define CR_ASYNC_TABLE_FULL 1        /* a frontier de-duplication table ran full */
#define CR_ASYNC_FRONTIER_OVERFLOW 2 /* a block's frontier needed more than cap_src entries (CR_SAMPLE_SMALL_FRONTIER) */

/*   device : the device the context's work runs on (informational; the caller selects devices)
 *   flags  : 0 or CR_CTX_DRY_RUN
 *   status : device int64[CR_CTX_STATUS_WORDS], caller-owned, zeroed by the caller, 8-byte aligned; NULL = kernels
 *            record overflows in the block headers only
 * Allocates host memory only. */
cr_status cr_ctx_create(cr_ctx **ctx, int32_t device, uint32_t flags, int64_t *status);
cr_status cr_ctx_destroy(cr_ctx *ctx);       /* frees host memory only; NULL is allowed */
/* Makes ctx (or none, with NULL) the calling thread's current context.  Other threads are not affected. */
cr_status cr_ctx_make_current(cr_ctx *ctx);
/* Reads the status words (one small copy on `stream`, then waits for that stream): CR_OK if nothing overflowed since
 * the words were last cleared, else CR_ERR_ASYNC_OVERFLOW with *required (may be NULL) = the largest frontier length
 * that was needed.  clear != 0 zeroes the words again (by a kernel on `stream`). */
cr_status cr_ctx_poll_error(cr_ctx *ctx, int64_t *required, int32_t clear, void *stream);

/* ------------------------------------------------------------------------- */
/* Step-1: root node partitioning (Algorithm 1 Step-1; Section 4.1; Table 1). */
/* ------------------------------------------------------------------------- */
enum {
    CR_ROOTS_NORAND = 0,    /* NORAND-ROOTS: training set as given, static across epochs */
    CR_ROOTS_COMM_RAND = 1, /* COMM-RAND-MIX: communities shuffled as blocks, mix_count of them merged
                               into a super-block, contents of each super-block shuffled */
    CR_ROOTS_RAND = 2       /* RAND-ROOTS: uniform shuffle of the whole training set */
};

typedef struct {
    int32_t policy;     /* CR_ROOTS_* */
    int32_t mix_count;  /* communities per super-block, >= 1 (1 = COMM-RAND-MIX-0%); ignored unless COMM_RAND */
    int32_t batch_size; /* > 0 */
    uint32_t epoch;     /* < 2^24 */
    uint64_t seed;
} cr_batch_cfg;

/* Number of communities per super-block for COMM-RAND-MIX-k%: k percent of the communities present
 * in the training set (Section 5, "Evaluated schemes"), rounded to nearest, at least 1. */
int32_t cr_mix_count_from_percent(double k_percent, int32_t n_comm_in_train);

cr_status cr_build_batches_workspace_bytes(int64_t n_train, int32_t n_comm, size_t *bytes /*host*/);

/* Writes the epoch's permutation of the training set; mini-batch b is
 * out_perm[b*batch_size .. min((b+1)*batch_size, n_train)) (the last batch may be short and is kept).
 *   train_ids : device int32[n_train], ascending and distinct (not checked on the device)
 *   comm      : device int32[n_nodes], community of every node, values in [0, n_comm)
 *   ws        : device workspace of at least cr_build_batches_workspace_bytes() bytes
 *   out_perm  : device int32[n_train]
 *   out_n_batches : host, may be NULL
 * Shuffles are "sort by a Philox4x32-10 key of (seed, epoch, id)", ties to the smaller id, so the
 * result is a pure function of the arguments.  n_train < 2^31. */
cr_status cr_build_batches(const cr_batch_cfg *cfg, const int32_t *train_ids, int64_t n_train,
                           const int32_t *comm, int32_t n_comm, void *ws, size_t ws_bytes,
                           int32_t *out_perm, int64_t *out_n_batches, void *stream);

/* cr_build_batches for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): the same result, bit for bit, with the sort buffers, digit histograms and
 * community tables in a fixed 8 MiB device array that belongs to the library instead of a caller workspace.  The call
 * allocates and frees nothing, on the host or on the device.
 *   limits : n_train <= CR_STATIC_MAX_TRAIN and n_comm <= CR_STATIC_MAX_COMM, otherwise CR_ERR_CAPACITY (use
 *            cr_build_batches with a workspace)
 *   sharing: every call on a GPU uses that GPU's one array (each GPU the library runs on holds its own copy until the
 *            process ends).  Nothing in it needs to start at zero from outside: the call clears what it accumulates
 *            into with a kernel of its own.  Two calls that overlap on one GPU (different streams or threads) race;
 *            calls on one stream, or ordered by events, are safe.
 * All other arguments as in cr_build_batches. */
#define CR_STATIC_MAX_TRAIN 262144
#define CR_STATIC_MAX_COMM 65536
cr_status cr_build_batches_static(const cr_batch_cfg *cfg, const int32_t *train_ids, int64_t n_train,
                                  const int32_t *comm, int32_t n_comm, int32_t *out_perm,
                                  int64_t *out_n_batches, void *stream);

/* ------------------------------------------------------------------------- */
/* Step-2: sub-graph construction (Algorithm 1 Step-2; Section 4.2).          */
/* ------------------------------------------------------------------------- */
typedef struct {
    int64_t n_nodes;
    int64_t n_entries;      /* = indptr[n_nodes] */
    const int64_t *indptr;  /* device int64[n_nodes+1] */
    const int32_t *indices; /* device int32[n_entries]; row v = neighbours of v (symmetrised graph) */
    const int32_t *comm;    /* device int32[n_nodes] */
    int32_t n_comm;
    int32_t reserved;
    const uint32_t *edge_intra; /* device uint32[ceil(n_entries/32)] or NULL: bit (e & 31) of word e >> 5 is set iff
                                   entry e joins two nodes of one community (filled by cr_graph_edge_classes).  Static
                                   per graph; lets biased sampling read a neighbour's class without touching
                                   indices[] and comm[].  Results are identical with and without it. */
} cr_graph;

/* Fills edge_intra (device uint32[ceil(n_entries/32)], every word fully written) from indptr / indices / comm;
 * graph->edge_intra itself is ignored here. */
cr_status cr_graph_edge_classes(const cr_graph *graph, uint32_t *edge_intra, void *stream);

/* The sampled blocks of ONE GNN layer for a group of n_batches mini-batches that are sampled
 * together.  Every array is laid out [n_batches][capacity]; batch g of the group owns slice g.
 * For batch g: rows 0..n_dst-1 are destination nodes; src_ids[0..n_src) are the global ids of the
 * frontier, whose first n_dst entries are the destination nodes themselves and whose remaining
 * entries are the newly reached neighbours in order of first appearance (rows ascending, adjacency
 * slot ascending); indptr/indices are a CSR over local source positions.  t_indptr/t_indices hold
 * the transposed block (for every source position the destination rows that use it, ascending);
 * they may be NULL when the layer's input needs no gradient, and must be NULL for layer 0 (the
 * feature table takes no gradient) unless CR_SAMPLE_TRANSPOSE_INPUT is set.  gather_ids is optional for every layer.
 * row_order is optional too: a processing order for the destination rows (see the field). */
typedef struct {
    int32_t n_batches;
    int32_t fanout;
    int32_t cap_dst;    /* rows per batch */
    int32_t cap_src;    /* frontier entries per batch */
    int32_t cap_nnz;    /* edges per batch = cap_dst * fanout */
    int32_t reserved;
    int32_t *hdr;       /* device int32[n_batches][CR_HDR_WORDS] */
    int32_t *src_ids;   /* device int32[n_batches][cap_src] */
    int32_t *indptr;    /* device int32[n_batches][cap_dst+1] */
    int32_t *indices;   /* device int32[n_batches][cap_nnz] */
    int32_t *t_indptr;  /* device int32[n_batches][cap_src+1] or NULL */
    int32_t *t_indices; /* device int32[n_batches][cap_nnz] or NULL */
    int32_t *gather_ids;/* device int32[n_batches][cap_nnz] or NULL: global id of every edge's source,
                           gather_ids[e] == src_ids[indices[e]]; lets the layer-0 feature gather skip one
                           level of indirection */
    int32_t *row_order; /* device int32[n_batches][cap_dst] or NULL: per batch a permutation of 0..n_dst-1.  Filled by
                           cr_sample_blocks (with CR_SAMPLE_ROW_ORDER) where it is given: destination rows grouped by the community of
                           their node
                           (communities ascending; the order inside a community is unspecified and may differ from run
                           to run).  cr_gather_aggregate_fwd and cr_gcn_aggregate_fwd walk the rows in this order, so
                           that rows which share source rows are worked on next to each other and meet in L1/L2 (the
                           locality Section 3 of the paper gets from the batch's composition, here from the order of
                           the work inside a batch).  A scheduling hint only: no result depends on it. */
    int32_t *group_order; /* device int32[n_batches*cap_dst + 1] or NULL: the same over the whole group of batches: entries
                           batch * cap_dst + row for every destination row of every batch, grouped by community (so the
                           rows of one community from all batches of the group are neighbours), followed, at index
                           n_batches*cap_dst, by their number.  Filled like row_order; read by
                           cr_gather_aggregate_fwd_group. */
} cr_block_set;

#define CR_SAMPLE_STRICT_INTRA 1u /* at p = 1 never take an inter-community neighbour (rows may be short) */
#define CR_SAMPLE_HASH_DEDUP 2u   /* de-duplicate the frontier with the open-addressing table even when the graph is small
                                     enough for the direct-address table (less workspace; same results) */

#define CR_SAMPLE_INPUT_GLOBAL_IDS 4u /* leave the input-side block (layer 0) in global ids: its frontier is not
                                     de-duplicated or relabelled.  Produced for layer 0: hdr (N_DST, NNZ, STATUS;
                                     N_SRC = -1), indptr, gather_ids (required) and src_ids[0..n_dst) (the destination
                                     nodes); src_ids beyond n_dst and indices are left untouched.  For a caller that
                                     reads the resident feature table through gather_ids and needs no gradient of the
                                     input features: the blocks of the layers above, and every result computed from
                                     them, are unchanged. */
#define CR_SAMPLE_TRANSPOSE_INPUT 8u /* layers[0] may carry t_indptr / t_indices too (a model whose first layer needs a
                                     gradient per source row: graph attention projects the source rows before it
                                     aggregates).  Not together with CR_SAMPLE_INPUT_GLOBAL_IDS. */

#define CR_SAMPLE_SMALL_FRONTIER 32u /* the block sets may be smaller than the bounds of cr_block_capacities (which assume that
                                  no two sampled neighbours of a batch coincide): per layer cap_src >= cap_dst, cap_nnz >=
                                  cap_dst * fanout, cap_dst of the root layer >= batch_size and cap_dst of layer l-1 >=
                                  min(cap_src of layer l, its bound).  A frontier that needs more than cap_src entries is
                                  cut at cap_src, its block (and what is sampled below it) gets a non-zero CR_HDR_STATUS, and
                                  the current context's status words record CR_ASYNC_FRONTIER_OVERFLOW with the length that
                                  was needed; every access stays inside the arrays.  The workspace is sized as without the
                                  flag. */

#define CR_SAMPLE_EXACT_RANKING 64u /* verification aid: neighbour selection without its pre-filter thresholds, every row ranked on
                                  full (key, slot) pairs -- the path that otherwise only serves the rare rows whose threshold
                                  let too few slots through or whose boundary keys are equal.  Same results, slower. */

#define CR_SAMPLE_ROW_ORDER 16u /* fill the row_order array of every layer whose block set carries one (the workspace is
                                  then larger: set the flag for cr_sample_blocks_workspace_bytes too) */

typedef struct {
    int32_t n_layers;              /* 1..CR_MAX_LAYERS */
    int32_t fanout[CR_MAX_LAYERS]; /* by GNN layer, 0 = input side; the roots are expanded with fanout[n_layers-1] */
    double p_intra;                /* [0.5, 1.0]: unnormalised weight of an intra-community edge; inter = 1 - p */
    uint64_t seed;
    uint32_t epoch;                /* < 2^24 */
    uint32_t first_batch;          /* index (within the epoch) of the group's first mini-batch */
    uint32_t flags;                /* CR_SAMPLE_* */
    uint32_t reserved;
} cr_sample_cfg;

/* Capacities that can never overflow for batches of at most batch_size roots:
 * cap_dst[L-1] = batch_size, cap_src[l] = min(n_nodes, cap_dst[l]*(1+fanout[l])), cap_dst[l-1] = cap_src[l]. */
cr_status cr_block_capacities(const cr_sample_cfg *cfg, int64_t n_nodes, int32_t batch_size,
                              int32_t *cap_dst /*host[n_layers]*/, int32_t *cap_src /*host[n_layers]*/,
                              int32_t *cap_nnz /*host[n_layers]*/);

cr_status cr_sample_blocks_workspace_bytes(const cr_sample_cfg *cfg, int64_t n_nodes, int32_t batch_size,
                                           int32_t n_batches, size_t *bytes /*host*/);

/* Which frontier de-duplication table cr_sample_blocks will use for this request (same results either way): one int32
 * per node and batch, addressed by node id (CR_DEDUP_DIRECT: graphs up to four times the largest table), or an
 * open-addressing table of twice the largest frontier (CR_DEDUP_HASH: larger graphs, or CR_SAMPLE_HASH_DEDUP). */
#define CR_DEDUP_DIRECT 0
#define CR_DEDUP_HASH 1
/* Self-test of the weighted neighbour selection (Section 4.2 with 0.5 < p < 1; exponential-clock keys): the selection
 * ranks single-precision keys first and accepts a row only if its result provably equals the one of the exact integer
 * keys, which rests on a bound on the error of the single-precision clock.  This call measures that error over all 2^32
 * random words on the device.  result: device float[4] (16-byte aligned), written asynchronously on `stream`:
 * [0] largest |error| in units of 2^-24 over the words of the upper half (clocks below 1), [1] largest relative error
 * over the lower half, [2] largest error as a fraction of the bound the library assumes (must be <= 1; the library keeps
 * a factor of two in hand), [3] zero.  ~30 ms.  Errors: CR_ERR_INVALID_ARG. */
cr_status cr_selftest_clock_approximation(float *result /*device*/, void *stream);

cr_status cr_sample_blocks_dedup_table(const cr_sample_cfg *cfg, int64_t n_nodes, int32_t batch_size, int32_t *kind /*host*/);

/* Samples the blocks of n_batches consecutive mini-batches in one set of launches.
 *   roots : device int32[n_roots_total]: the slice of the epoch's permutation that starts at
 *           mini-batch cfg->first_batch; batch g of the group is roots[g*batch_size ..
 *           min((g+1)*batch_size, n_roots_total)); only the last may be short
 *   layers: host array [n_layers] of block sets with n_batches == n_batches, fanout == cfg->fanout[l]
 *           and capacities >= cr_block_capacities()
 * For every destination row v with d neighbours, adjacency slot j gets the word
 * Philox4x32-10(seed; slot>>2, v, batch, epoch<<8|2<<4|layer)[slot&3] and an integer key that orders
 * the slots like independent exponential clocks of rate p (intra) or 1-p (inter); the
 * min(fanout, d) smallest (key, slot) pairs are kept.  The output is a pure function of the
 * arguments (bit-reproducible). */
cr_status cr_sample_blocks(const cr_graph *graph, const cr_sample_cfg *cfg, const int32_t *roots,
                           int64_t n_roots_total, int32_t batch_size, int32_t n_batches, void *ws,
                           size_t ws_bytes, cr_block_set *layers, void *stream);

/* ------------------------------------------------------------------------- */
/* Training on the sub-graph: message passing of Eq. 1 in GraphSAGE-mean form */
/*   Agg[v] = mean_{u in N_s(v)} H[u]   (0 for an empty row)                  */
/*   Z[v]   = H[v] W_self + Agg[v] W_neigh + b ; ReLU on hidden layers        */
/* ------------------------------------------------------------------------- */
enum { CR_F32 = 0, CR_BF16 = 1 };

/* Feature-row gather with mean aggregation for batch g of a block set (the input-feature fetch the
 * paper identifies as the cost that tracks the batch's footprint, Section 6.1.1).
 *   H_src    : device; indirect != 0: the resident feature table [n_nodes][ld_src], row of local
 *              source position s is src_ids[s] (read through blocks->gather_ids when that is given);
 *              indirect == 0: dense [n_src][ld_src]
 *   dtype    : CR_F32 or CR_BF16 element type of H_src;  F <= 1024 columns
 *   agg      : device float [cap_dst][F] or NULL
 *   agg_bf16 : device bf16 [cap_dst][ld_bf16] or NULL; columns F..ld_bf16-1 are written as zero
 *   self_bf16: device bf16 [cap_dst][ld_bf16] or NULL; row v = H_src row of destination v (same padding)
 *   ld_bf16  : multiple of 32, >= F, <= F rounded up to 64
 * Rows >= n_dst (read from the block header on the device) are not touched. */
cr_status cr_gather_aggregate_fwd(const cr_block_set *blocks, int32_t g, const void *H_src,
                                  int32_t dtype, int64_t ld_src, int32_t F, int32_t indirect,
                                  float *agg, uint16_t *agg_bf16, uint16_t *self_bf16,
                                  int64_t ld_bf16, void *stream);

/* The same for every batch of the group in one launch (indirect addressing through blocks->gather_ids, bf16 outputs
 * only): the input features take no gradient and no weight enters here, so the aggregation of a whole sampled group
 * can run ahead of the training steps, and walking blocks->group_order (required) puts the rows of one community from
 * all batches next to each other: a feature row is then fetched once for the group rather than once per batch.
 *   agg_bf16, self_bf16 : device bf16 [n_batches][batch_stride_rows][ld_bf16]; batch g's rows start at row
 *                         g * batch_stride_rows (>= cap_dst); same contents as cr_gather_aggregate_fwd writes */
cr_status cr_gather_aggregate_fwd_group(const cr_block_set *blocks, const void *H_src, int32_t dtype, int64_t ld_src,
                                        int32_t F, uint16_t *agg_bf16, uint16_t *self_bf16, int64_t batch_stride_rows,
                                        int64_t ld_bf16, void *stream);

/* Backward of the aggregation w.r.t. the source rows, atomic-free over the transposed block:
 *   d_src[u] = sum_{v : u in N_s(v)} d_agg[v] / |N_s(v)|   (+ d_self[u] for u < n_dst)
 *   d_agg, d_self : device float or bf16 (in_dtype) [cap_dst][ld_in] (d_self may be NULL); ld_in a multiple of 4
 *                   (float) or 8 (bf16); sums are accumulated in float either way
 *   d_src         : device float [cap_src][F] or NULL, rows 0..n_src-1 fully overwritten
 *   relu_out      : device float or bf16 (relu_dtype) [cap_src][ld_relu] or NULL: forward output of the layer
 *                   below; where it is <= 0 the gradient is zeroed (ReLU backward)
 *   d_src_bf16    : device bf16 [cap_src][ld_bf16] or NULL (same masking, zero padded columns) */
cr_status cr_gather_aggregate_bwd(const cr_block_set *blocks, int32_t g, const void *d_agg,
                                  const void *d_self, int32_t in_dtype, int64_t ld_in, int32_t F,
                                  const void *relu_out, int32_t relu_dtype, int64_t ld_relu, float *d_src,
                                  uint16_t *d_src_bf16, int64_t ld_bf16, void *stream);

/* ------------------------------------------------------------------------- */
/* GCN on the same blocks (Section 6.4: the method generalises to other models; Kipf & Welling's propagation rule     */
/* with the renormalisation trick, d~ = degree in the full graph + 1):                                                 */
/*   exact : out[v] = sum_{u in N(v) + {v}} H[u] / sqrt(d~_v d~_u)                                                     */
/*   block : out[v] = H[v] / d~_v + (deg_v / |N_s(v)|) / sqrt(d~_v) * sum_{u in N_s(v)} H[u] / sqrt(d~_u)              */
/* (the neighbour sum is estimated from the sampled neighbours; exact when all were taken, unbiased under uniform       */
/* sampling).  The dense part is a one-operand layer, Z = out W + b.                                                    */
/* ------------------------------------------------------------------------- */
/* norm: device float[2*n_nodes], norm[2v] = 1/sqrt(d~_v), norm[2v+1] = deg_v; static per graph. */
cr_status cr_graph_gcn_norm(const cr_graph *graph, float *norm, void *stream);

/* Per-batch normalisation of block g: blk_norm is a device float[cap_src + 2*cap_dst] scratch that the two calls below
 * read (source weights, destination scales, destination self weights); compute it once per sampled block and batch. */
cr_status cr_gcn_block_norm(const cr_block_set *blocks, int32_t g, const float *norm, float *blk_norm, void *stream);

/* Arguments as cr_gather_aggregate_fwd (no self output: the destination's own row is part of the sum).  indirect != 0
 * needs blocks->gather_ids. */
cr_status cr_gcn_aggregate_fwd(const cr_block_set *blocks, int32_t g, const float *norm, const float *blk_norm,
                               const void *H_src, int32_t dtype, int64_t ld_src, int32_t F, int32_t indirect,
                               float *agg, uint16_t *agg_bf16, int64_t ld_bf16, void *stream);

/* cr_gcn_aggregate_fwd for every batch of the group in one launch (input-side block, indirect addressing through
 * blocks->gather_ids, bf16 output only), walking blocks->group_order like cr_gather_aggregate_fwd_group; rows wider than
 * 1 KB go in column panels there as here.  The destination scales and self weights are taken from `norm` directly, so
 * no cr_gcn_block_norm is needed for this block.  Same bits as the per-batch call.
 *   agg_bf16 : device bf16 [n_batches][batch_stride_rows][ld_bf16] */
cr_status cr_gcn_aggregate_fwd_group(const cr_block_set *blocks, const float *norm, const void *H_src, int32_t dtype,
                                     int64_t ld_src, int32_t F, uint16_t *agg_bf16, int64_t batch_stride_rows,
                                     int64_t ld_bf16, void *stream);

/* Transpose of cr_gcn_aggregate_fwd (dense addressing): gradient with respect to the source rows, atomic-free over the
 * transposed block.  d_out: device float or bf16 (in_dtype) [cap_dst][ld_in]; other arguments as
 * cr_gather_aggregate_bwd. */
cr_status cr_gcn_aggregate_bwd(const cr_block_set *blocks, int32_t g, const float *blk_norm, const void *d_out,
                               int32_t in_dtype, int64_t ld_in, int32_t F, const void *relu_out, int32_t relu_dtype,
                               int64_t ld_relu, float *d_src, uint16_t *d_src_bf16, int64_t ld_bf16, void *stream);

/* ------------------------------------------------------------------------- */
/* Graph attention on the same blocks (Section 6.4 names GAT as the second other model; the layer is the one of         */
/* Velickovic et al., "Graph Attention Networks"):                                                                      */
/*   z[u]      = x[u] W                       a one-operand layer without bias over the block's SOURCE rows             */
/*   e[v,u,h]  = LeakyReLU_slope(a_l[h] . z[u,h] + a_r[h] . z[v,h])   for u in N_s(v), head h = columns h*D..h*D+D-1    */
/*   alpha     = softmax of e over N_s(v)     (sampled in-neighbours, no added self loop)                               */
/*   out[v,h]  = sum_u alpha[v,u,h] z[u,h] + bias[h]     (ReLU on hidden layers; a row without neighbours: the bias)    */
/* The projection and its backward are cr_sage_linear_fwd / cr_sage_linear_bwd on a layer with n_operands = 1 and       */
/* bias = NULL, run over the source rows (header + CR_HDR_N_SRC); the calls below are the attention part.               */
/* ------------------------------------------------------------------------- */
typedef struct {
    int32_t heads, D;  /* heads * D = the layer's F_out; with several heads D must be 8 times a power of two */
    float slope;       /* negative slope of the LeakyReLU, in [0, 1] */
    int32_t reserved;
    float *attn;       /* device float [3][ld]: a_l, a_r and the bias by output column (ld = the layer's N_pad; entries
                          >= heads*D must be 0) */
} cr_gat_params;

/* rows_out[i] = store[ids[i]] converted to bf16 and zero padded to ld_out columns, for i < n = min(hdr[hdr_word],
 * max_n): the first layer's projection operand (one row per distinct input node of the batch).
 *   store : device [n_nodes][ld_src] of CR_F32 or CR_BF16, F real columns;  rows_out : device bf16 [max_n][ld_out] */
cr_status cr_gather_rows_bf16(const void *store, int32_t dtype, int64_t ld_src, int32_t F, const int32_t *ids,
                              const int32_t *hdr, int32_t hdr_word, int32_t max_n, uint16_t *rows_out,
                              int64_t ld_out, void *stream);

/* Attention scores, neighbourhood softmax and weighted sum for batch g.
 *   z_bf16 : device bf16 [cap_src][ld], the projected source rows (padded columns zero); ld = 64..512, multiple of 64
 *   el, er : device float [cap_src][heads]: written (the two halves of every score)
 *   stat   : device float [cap_dst][heads][4], 16-byte aligned: written; per destination and head what the backward
 *            pass needs to recompute alpha (er, largest score, 1 / sum of exponentials, one word for its own use)
 *   out    : device float [cap_dst][ld] or NULL;  out_bf16 : device bf16 [cap_dst][ld] or NULL */
cr_status cr_gat_attention_fwd(const cr_block_set *blocks, int32_t g, const cr_gat_params *params,
                               const uint16_t *z_bf16, int64_t ld, int32_t relu, float *el, float *er,
                               float *stat, float *out, uint16_t *out_bf16, void *stream);

cr_status cr_gat_attention_bwd_workspace_bytes(int32_t cap_dst, int64_t ld, int32_t heads, size_t *bytes);

/* Backward of cr_gat_attention_fwd and one SGD step on a_l, a_r (with weight decay) and the bias (without).  Needs the
 * transposed block (for layer 0: sample with CR_SAMPLE_TRANSPOSE_INPUT); no atomics, bit-reproducible.
 *   z_bf16, el, stat : as left by the forward call of the same batch (stat's spare word is overwritten)
 *   d_out_bf16    : device bf16 [cap_dst][ld_dout]: dL/d out (after the ReLU, if any)
 *   relu_out_bf16 : device bf16 [cap_dst][ld] or NULL: the forward output; where it is <= 0 the gradient is zeroed
 *   dz_bf16       : device bf16 [cap_src][ld]: dL/dz for rows 0..n_src-1 (the dz operand of cr_sage_linear_bwd)
 *   d_attn_out    : device float [3][ld] or NULL: the gradients of a_l, a_r and the bias
 *   ws            : device workspace of cr_gat_attention_bwd_workspace_bytes(cap_dst, ld, heads) bytes */
cr_status cr_gat_attention_bwd(const cr_block_set *blocks, int32_t g, const cr_gat_params *params,
                               const uint16_t *z_bf16, int64_t ld, const float *el, float *stat,
                               const uint16_t *d_out_bf16, int64_t ld_dout, const uint16_t *relu_out_bf16,
                               float lr, float weight_decay, uint16_t *dz_bf16, float *d_attn_out, void *ws,
                               size_t ws_bytes, void *stream);

/* One layer's dense parameters.  F_pad = F_in rounded up to 32, N_pad = F_out rounded up to 64.
 * n_operands = 2: GraphSAGE, Z = H_self W_self + Agg W_neigh + b;  n_operands = 1: one aggregated input (GCN,
 * Section 6.4), Z = Agg W + b: every h_self / d_self argument below must then be NULL and the [.. 2*F ..] shapes
 * read [.. F ..]. */
typedef struct {
    int32_t F_in, F_out;
    int32_t n_operands; /* 1 or 2 */
    int32_t reserved;
    float *W;          /* device float [n_operands*F_in][F_out]: rows 0..F_in-1 = W_self, F_in..2F_in-1 = W_neigh (master) */
    float *bias;       /* device float [N_pad] (entries >= F_out stay 0), or NULL: a layer without a bias term (none added,
                          none updated) */
    uint16_t *W_bf16;  /* device bf16 [n_operands*F_pad][N_pad], zero padded shadow of W (row F_pad+k = W_neigh row k) */
    uint16_t *Wt_bf16; /* device bf16 [N_pad][n_operands*F_pad], its transpose */
} cr_sage_layer;

cr_status cr_sage_padded_dims(int32_t F_in, int32_t F_out, int32_t *F_pad, int32_t *N_pad);
/* Rebuilds both bf16 shadows from the float master (call once after initialising W). */
cr_status cr_sage_refresh_shadows(const cr_sage_layer *layer, void *stream);

/* out[v] = h_self[v] W_self + agg[v] W_neigh + bias (ReLU if relu != 0), bf16 operands on the matrix
 * cores with float accumulation.
 *   hdr     : device block header; rows = hdr[CR_HDR_N_DST]; max_rows bounds the launch.  Only that one word is read,
 *             so a product over a block's source rows (the graph-attention projection) passes header + CR_HDR_N_SRC
 *   h_self, agg : device bf16 [max_rows][ld_in], ld_in >= F_pad, padded columns zero
 *   out     : device float [max_rows][N_pad] or NULL;  out_bf16 : device bf16 [max_rows][N_pad] or NULL */
cr_status cr_sage_linear_fwd(const cr_sage_layer *layer, const int32_t *hdr, int32_t max_rows,
                             const uint16_t *h_self, const uint16_t *agg, int64_t ld_in, int relu,
                             float *out, uint16_t *out_bf16, void *stream);

cr_status cr_sage_linear_bwd_workspace_bytes(int32_t F_in, int32_t F_out, int32_t max_rows, size_t *bytes);

/* Backward of cr_sage_linear_fwd followed by one SGD step W <- W - lr*(dW + weight_decay*W),
 * b <- b - lr*db on the master weights; both bf16 shadows are refreshed.
 *   dz_bf16 : device bf16 [max_rows][N_pad]: dL/dZ with the ReLU mask already applied, padded columns zero
 *   d_self, d_agg : device float [max_rows][F_pad] or both NULL; computed with the weights from before the step
 *   d_in_bf16 : device bf16 [max_rows][2*F_pad] or NULL: the same input gradients rounded to bf16 (nearest even),
 *               d_self in columns 0..F_pad-1, d_agg in F_pad..2*F_pad-1.  With all three NULL no input gradient
 *               is computed (layer 0: the features need none)
 *   dW_out  : device float [2*F_in][F_out] or NULL, db_out: device float [F_out] or NULL: the gradients
 *   ws      : device workspace of cr_sage_linear_bwd_workspace_bytes() bytes */
cr_status cr_sage_linear_bwd(const cr_sage_layer *layer, const int32_t *hdr, int32_t max_rows,
                             const uint16_t *h_self, const uint16_t *agg, int64_t ld_in,
                             const uint16_t *dz_bf16, float lr, float weight_decay, float *d_self,
                             float *d_agg, uint16_t *d_in_bf16, float *dW_out, float *db_out, void *ws,
                             size_t ws_bytes, void *stream);

/* Only the input gradients of cr_sage_linear_bwd (d_self = dZ W_self^T, d_agg = dZ W_neigh^T; float pair and/or
 * the bf16 array, as there; at least one of the two forms); no weight is touched.  Lets a caller put the
 * weight-gradient part (cr_sage_linear_bwd without input gradients) on another stream, off the critical path of
 * the backward pass; that call must then be ordered after this one, which reads the weights from before the step. */
cr_status cr_sage_linear_bwd_input(const cr_sage_layer *layer, const int32_t *hdr, int32_t max_rows,
                                   const uint16_t *dz_bf16, float *d_self, float *d_agg, uint16_t *d_in_bf16,
                                   void *stream);

/* Backward pass of one whole GraphSAGE-mean layer above the input layer (Eq. 1, differentiated) in two launches
 * instead of four.  Same results, bit for bit, as
 *   cr_sage_linear_bwd(layer, header of batch g, blocks->cap_dst, h_self, agg, ld_in, dz_bf16, lr, weight_decay,
 *                      NULL, NULL, d_in_bf16, dW_out, db_out, ws, ws_bytes)
 * followed by
 *   cr_gather_aggregate_bwd(blocks, g, d_agg = d_in_bf16 + F_pad, d_self = d_in_bf16, CR_BF16, 2*F_pad, layer->F_in,
 *                           relu_out_bf16, CR_BF16, ld_relu, NULL, d_src_bf16, ld_bf16):
 * the first launch holds the two products (weight gradient, input gradient), the second the aggregation's backward
 * pass together with the reduction + SGD step of the weights; the members of each pair need nothing from each other.
 *   layer         : a two-operand layer;  blocks : needs the transposed block
 *   d_in_bf16     : device bf16 [cap_dst][2*F_pad], scratch that holds the layer's input gradients afterwards
 *   relu_out_bf16 : device bf16 [cap_src][ld_relu] or NULL, forward output of the layer below (ReLU mask)
 *   d_src_bf16    : device bf16 [cap_src][ld_bf16]: dL/dZ of the layer below
 * Everything else as in the two calls above. */
cr_status cr_sage_layer_bwd(const cr_sage_layer *layer, const cr_block_set *blocks, int32_t g,
                            const uint16_t *h_self, const uint16_t *agg, int64_t ld_in, const uint16_t *dz_bf16,
                            float lr, float weight_decay, uint16_t *d_in_bf16, const uint16_t *relu_out_bf16,
                            int64_t ld_relu, uint16_t *d_src_bf16, int64_t ld_bf16, float *dW_out, float *db_out,
                            void *ws, size_t ws_bytes, void *stream);

/* Mean softmax cross-entropy over the root rows (labels exist for roots only) and its gradient.
 *   hdr      : device block header of the root block; n = hdr[CR_HDR_N_DST] <= max_rows
 *   logits   : device float [max_rows][ld], only columns 0..n_classes-1 take part
 *   labels   : device int32[n_nodes] indexed by global node id;  root_ids : device int32[>= n]
 *   loss     : device float[1];  row_loss : device float [max_rows] scratch
 *   d_logits : device float [max_rows][ld] or NULL;  d_logits_bf16 : device bf16 [max_rows][ld] or NULL
 *              (columns >= n_classes written as zero) */
cr_status cr_softmax_xent(const int32_t *hdr, int32_t max_rows, const float *logits, int64_t ld,
                          int32_t n_classes, const int32_t *labels, const int32_t *root_ids,
                          float *loss, float *row_loss, float *d_logits, uint16_t *d_logits_bf16,
                          void *stream);

/* The layer next to the loss and the loss in one call: cr_sage_linear_fwd(relu = 0, out = logits, out_bf16 = NULL)
 * followed by cr_softmax_xent(hdr, max_rows, logits, N_pad, n_classes, ..., d_logits = NULL, d_logits_bf16).  When the
 * layer has at most 64 outputs and the block at most 2048 rows (by max_rows) this is one launch: a workgroup of the
 * product holds whole rows of logits and finishes their loss terms in place; otherwise the separate kernels run.
 * Logits are bit-identical to cr_sage_linear_fwd's; the loss terms may differ from cr_softmax_xent's in the last
 * bits (sums are associated differently), never from run to run.
 *   logits        : device float [max_rows][N_pad];  d_logits_bf16 : device bf16 [max_rows][N_pad]
 *   scratch       : device, CR_XENT_SCRATCH_BYTES; zero before the first call, and every call leaves it zero again;
 *                   calls that share a scratch must not overlap.  In the one-launch form the mean loss is the sum of
 *                   per-workgroup shares rounded to 2^-20 (a device-side integer accumulator: reproducible whatever the
 *                   order of arrival), NaN if a share is not finite
 * The remaining arguments as in the two calls. */
#define CR_XENT_SCRATCH_BYTES 512
cr_status cr_sage_linear_fwd_xent(const cr_sage_layer *layer, const int32_t *hdr, int32_t max_rows,
                                  const uint16_t *h_self, const uint16_t *agg, int64_t ld_in, float *logits,
                                  int32_t n_classes, const int32_t *labels, const int32_t *root_ids, float *loss,
                                  float *row_loss, uint16_t *d_logits_bf16, void *scratch, void *stream);

/* Validation pass of the training protocol (Section 5 "Training methodology": final validation accuracy, early
 * stopping on the validation loss): adds to *count the number of root rows whose largest logit (lowest class index
 * on ties) equals the label.  Same arguments as cr_softmax_xent; count is a device int32 that the caller zeroes.
 * The validation loss comes from cr_softmax_xent with both gradient outputs NULL. */
cr_status cr_count_correct(const int32_t *hdr, int32_t max_rows, const float *logits, int64_t ld,
                           int32_t n_classes, const int32_t *labels, const int32_t *root_ids,
                           int32_t *count, void *stream);

/* Mean of a per-batch mean over batches of different sizes (the validation loss of the training protocol is the mean
 * over all validation nodes, and the last batch is short): with n = min(hdr[CR_HDR_N_DST], max_rows),
 *   acc[0] += value[0] * n,  acc[1] += n,  acc[2] = acc[0] / acc[1].
 *   value : device float[1] (the loss cr_softmax_xent left for this batch)
 *   acc   : device double[3], zeroed by the caller before the first batch; calls must be ordered (one stream) */
cr_status cr_mean_accumulate(const int32_t *hdr, int32_t max_rows, const float *value, double *acc, void *stream);

/* ------------------------------------------------------------------------- */
/* Software-managed feature cache (Section 6.5, impact of software-managed     */
/* caches: feature rows kept in a slower store, an LRU cache of rows in GPU    */
/* memory in front of it).                                                     */
/* ------------------------------------------------------------------------- */
/* Set-associative (set = node id mod n_sets, `ways` rows per set), updated once per mini-batch:
 *   1. every distinct input node of the batch is looked up; a hit refreshes its row's stamp;
 *   2. the misses of a set, in the order the nodes appear in the batch, replace that set's rows in order of
 *      (stamp ascending, way ascending), never a row hit or filled in this batch (empty rows have stamp -1);
 *   3. misses that find no such row are copied to a per-batch overflow area behind the cached rows instead (the
 *      node at position i of the batch to overflow row i).
 * After a fetch, rows[slot_out[i]] holds the feature row of ids[i] for every i, so the feature gather can read the
 * cache's row array through slot_out in place of the store through the node ids.  All arrays are the caller's. */
#define CR_CACHE_MAX_WAYS 64
#define CR_CACHE_LIST_CAP 64 /* entries of a set's scratch list (the earliest CR_CACHE_MAX_WAYS misses of the batch) */

typedef struct {
    int32_t n_sets;     /* >= 1 */
    int32_t ways;       /* 1..CR_CACHE_MAX_WAYS */
    int32_t row_bytes;  /* bytes per feature row, multiple of 16 */
    int32_t n_overflow; /* rows of the overflow area, >= the largest batch's number of distinct input nodes */
    int32_t *keys;      /* device int32[n_sets*ways]: node id, or -1 */
    int32_t *stamps;    /* device int32[n_sets*ways]: stamp of the last batch that used the row, or -1 */
    void *rows;         /* device [(n_sets*ways + n_overflow)][row_bytes], 16-byte aligned */
    int32_t *set_count; /* device int32[n_sets]: scratch, zero between calls */
    int32_t *set_list;  /* device int32[n_sets][CR_CACHE_LIST_CAP]: scratch, kept by cr_cache_reset / cr_cache_fetch */
    int32_t *counters;  /* device int32[8], cumulative since cr_cache_reset: [0] look-ups, [1] misses, [2] misses that
                           went to the overflow area (any number of misses per set and batch is handled); [3..7]
                           unused, zero */
} cr_feature_cache;

/* Empties the cache and zeroes its scratch and counters. */
cr_status cr_cache_reset(const cr_feature_cache *cache, void *stream);

/* One batch's look-ups and replacements.
 *   store     : the feature store, [n_nodes][store_ld_bytes] bytes, readable by the GPU: device memory, or host memory
 *               from cr_host_alloc (its device_ptr); only the rows of missing nodes are read, once each
 *   ids       : device int32[>= n]: the batch's distinct input nodes; n = min(hdr[hdr_word], max_n) read on the device
 *               (a block header with hdr_word = CR_HDR_N_SRC, or any device int32)
 *   stamp     : the batch's stamp, increasing from batch to batch, >= 0
 *   slot_out  : device int32[max_n]: row of `rows` that holds ids[i]'s features */
cr_status cr_cache_fetch(const cr_feature_cache *cache, const void *store, int64_t store_ld_bytes,
                         const int32_t *ids, const int32_t *hdr, int32_t hdr_word, int32_t max_n,
                         int32_t stamp, int32_t *slot_out, void *stream);

/* The store without a cache: copies the rows of the batch's distinct input nodes, rows_out[i] = store[ids[i]] for
 * i < n = min(hdr[hdr_word], max_n), each row read once (what a unified-addressing gather of the input features
 * does); the feature gather then reads rows_out as a dense [n_src][row_bytes] array (indirect = 0).
 *   rows_out : device [max_n][row_bytes], 16-byte aligned; row_bytes a multiple of 16 */
cr_status cr_stage_rows(const void *store, int64_t store_ld_bytes, const int32_t *ids, const int32_t *hdr,
                        int32_t hdr_word, int32_t max_n, void *rows_out, int32_t row_bytes, void *stream);

/* Pinned host memory that kernels can read (for a feature store that stays on the host, as in the paper's
 * mixed CPU+GPU set-up for its largest graph).  *host_ptr is the address for the CPU, *device_ptr the one for
 * kernels.  Synchronous; free with cr_host_free(host_ptr). */
cr_status cr_host_alloc(size_t bytes, void **host_ptr, void **device_ptr);
cr_status cr_host_free(void *host_ptr);

#ifdef __cplusplus
}
#endif
#endif /* COMMRAND_H */
