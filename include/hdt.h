/*
 * hdt.h -- C ABI of the hierarchical document attention library for AMD MI355X (gfx950).
 *
 * The library computes the sparse attention of the Hierarchical Document Transformer
 * (arXiv 2407.08330, Sec. 3.2 "Hierarchical Attention" and App. A.1, Alg. 1):
 *
 *     A = Q K^T * softmax_scale,   S = softmax(A masked by M),   O = S V
 *
 * where every position of a document is a regular token or an auxiliary anchor
 * ([DOC], [SEC], [SENT], or any deeper hierarchy) and M lets a position attend only to
 * its parent, its siblings (itself included) and its children.  M differs per sample and is
 * shared by all heads.  M is never materialised: hdt_build_layout turns the per-position
 * `level` and `parent` ids into a block-sparse tile schedule, and the attention calls walk
 * that schedule.
 *
 * Conventions for every entry point
 *   - Pointers named d_* and all tensor pointers are DEVICE pointers owned by the caller;
 *     pointers named h_* are HOST pointers.  The library never takes ownership of them.
 *   - Tensors are dense and contiguous: Q, K, V, O, dO, dQ, dK, dV are [batch][heads][n_pos]
 *     [head_dim]; LSE is [batch][heads][n_pos] float; level, parent are [batch][n_pos] int32.
 *     Tensor base pointers must be 16-byte aligned.  Outputs must not alias inputs.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Attention calls
 *     only enqueue work on it; they never synchronise and never allocate.
 *   - Every function returns an hdt_status_t; nothing aborts or throws across the boundary.
 *     hdt_last_error() gives a thread-local text for the last non-OK status.
 *   - Rows of pad positions may hold anything, NaN and infinities included: no result at a real
 *     position depends on them, and their own output rows are written as stated below.  The same
 *     holds for the K, V rows of encoder positions a cross-attention layout does not make visible.
 *     A masked pair contributes nothing (Sec. 3.2), whatever the two rows hold.
 */
#ifndef HDT_H
#define HDT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    HDT_OK = 0,
    HDT_ERR_INVALID_ARG = 1, /* NULL pointer, negative size, non-positive or non-finite scale */
    HDT_ERR_SHAPE = 2,       /* sizes inconsistent with the layout or out of the supported range */
    HDT_ERR_HIERARCHY = 3,   /* level/parent arrays do not describe a valid hierarchy */
    HDT_ERR_UNSUPPORTED = 4, /* head_dim, dtype or tile shape without a kernel */
    HDT_ERR_OOM = 5,         /* device or host allocation failed */
    HDT_ERR_HIP = 6          /* a HIP runtime call failed (text in hdt_last_error) */
} hdt_status_t;

typedef enum {
    HDT_BF16 = 0, /* bf16 tensors, fp32 accumulation, MFMA kernels                */
    HDT_F32 = 1   /* fp32 tensors, plain fp32 arithmetic: the slow debugging path */
} hdt_dtype_t;

/* Level id of a pad position; anchors and tokens carry levels 0 .. HDT_MAX_LEVELS-1
 * (0 = the root, e.g. [DOC]=0, [SEC]=1, [SENT]=2, token=3). */
#define HDT_LEVEL_PAD (-1)
#define HDT_MAX_LEVELS 32

/* Kinds of hierarchy edges that carry attention (hdt_layout_opts_t.edges).  All three together are the
 * pattern of Sec. 3.2; the paper's ListOps study (Sec. 4.1) thins it: HDT_EDGE_SIBLING | HDT_EDGE_DOWN
 * ("operands do not attend to their operators") and HDT_EDGE_DOWN alone ("nor to each other").  A
 * position always attends to itself.  Without HDT_EDGE_UP == HDT_EDGE_DOWN symmetry the mask is directed;
 * the layout then also holds the schedule of the transposed mask, which the backward pass needs. */
#define HDT_EDGE_UP 1      /* a position attends to its parent   */
#define HDT_EDGE_SIBLING 2 /* a position attends to its siblings */
#define HDT_EDGE_DOWN 4    /* a position attends to its children */
#define HDT_EDGE_ALL 7

typedef struct hdt_layout hdt_layout_t; /* opaque; owns its device buffers */

typedef struct {
    int32_t tile_m;      /* query rows per tile,  0 = default (128); multiple of 32, <= 128   */
    int32_t tile_n;      /* key slots per tile,   0 = default (64);  multiple of 32, <= 128   */
    int32_t force_dense; /* 1: issue every tile (dense masked-attention baseline)             */
    int32_t no_sort;     /* 1: keep keys in document order (block-sparse baseline w/o sort)   */
    int32_t windowed;    /* 1: key tiles are fixed windows of the key order (Alg. 1 as printed); */
                         /* 0: every query tile gets its own packed key list (default)         */
    int32_t edges;       /* OR of HDT_EDGE_*; 0 = HDT_EDGE_ALL                                  */
    int32_t deferred;    /* 1: hdt_build_layout does not wait for the device (see there); key lists only */
    int32_t reserved;    /* 0 */
    int64_t capacity;    /* list entries the layout has room for; 0 = the library chooses        */
} hdt_layout_opts_t;

typedef struct {
    int32_t batch, n_pos, tile_m, tile_n;
    int32_t q_tiles, k_tiles; /* per sample: ceil(n_pos/tile_m), ceil(n_pos/tile_n)  */
    int32_t windowed;         /* 1: fixed key windows, 0: per-query-tile key lists   */
    int32_t edges;            /* OR of HDT_EDGE_* the mask was built with            */
    int64_t n_tiles;          /* surviving tiles (list entries), summed over the batch */
    int64_t nnz;              /* allowed (query, key) pairs, summed over the batch   */
    int64_t device_bytes;     /* device memory held by the layout                    */
    int32_t n_kv;             /* rows per sample of the gathered tensors (K, V in the forward): n_pos for a
                                 self-attention layout, the encoder length for a cross-attention layout */
    int32_t cross;            /* 1: built by hdt_build_cross_layout                  */
    uint32_t cross_level_mask;
    int32_t compact_rows;     /* cross-attention layout whose backward runs on compact copies of K and V: their
                                 rows per sample; 0 otherwise (see hdt_build_cross_layout)              */
} hdt_layout_info_t;

/*
 * hdt_build_layout -- level/parent ids -> block-sparse tile schedule, built on the device.
 * (Sec. 3.2: mask definition; App. A.1, Alg. 1: "sort K, V according to the hierarchy level",
 * partition into blocks, process only blocks with a non-zero mask entry.)
 *
 *   d_level  [batch][n_pos] int32, device: hierarchy level of each position, HDT_LEVEL_PAD for pads
 *   d_parent [batch][n_pos] int32, device: index (inside the same sample) of the parent position,
 *            -1 for a root and for pads.  Any forest is accepted; positions need not be in
 *            pre-order (documents laid out with anchors prepended give the fewest tiles).
 *   opts     host, may be NULL (all defaults)
 *   out      receives the layout; destroy it with hdt_layout_destroy
 *
 * The schedule, per sample:
 *   kperm    key order: positions sorted by level (0, 1, 2, ...; pads last), ties in document order
 *            (document order throughout with no_sort);
 *   allowed(i, j) = both non-pad and (i == j, or parent[i] == parent[j] >= 0 [HDT_EDGE_SIBLING], or
 *            parent[i] == j [HDT_EDGE_UP], or parent[j] == i [HDT_EDGE_DOWN]), the bracketed kinds as enabled
 *            by opts->edges;
 *   a tile = tile_m consecutive query rows [I*tile_m, (I+1)*tile_m) in document order x tile_n keys.
 *   windowed = 1 (Alg. 1 as printed): the keys of tile (I, J) are the slots [J*tile_n, (J+1)*tile_n)
 *            of the key order; the tile survives iff some pair in it is allowed; the tiles of a
 *            query tile are listed with J ascending.
 *   windowed = 0 (default): query tile I lists U_I = { j : some row of the tile may attend to j } in
 *            key order and cuts that list into tiles of tile_n keys (the last one filled up with
 *            "no key"); no tile is empty and no key without an allowed pair is ever gathered.  This is
 *            the same partition of the same mask with fewer, fuller tiles (the paper's closing remark
 *            of Sec. 3.2 leaves better permutations open); the attention results are identical.
 *   per tile: the document position behind each of its tile_n key slots, a bitmap of the allowed
 *            pairs and a summary of its 32x32 sub-blocks.  force_dense implies windowed.
 *
 * Enqueues kernels on `stream` and returns as soon as the first of them has reported, through pinned
 * host memory, that the hierarchy is valid and how many tiles the lists need: the call waits for that
 * kernel (and for whatever was enqueued on `stream` before it), not for the stream.  The rest of the
 * build may still be running when the call returns; work enqueued on the same stream afterwards is
 * ordered behind it, work on other streams must wait for `stream` first.  Device memory for the
 * layout comes from a cache of buffers of destroyed layouts (hipMalloc when the cache has nothing
 * that fits).  batch == 0 or n_pos == 0 gives an empty layout on which the attention calls are no-ops.
 *
 * opts->deferred = 1 (key-list layouts; ignored for windowed and dense ones): the call only enqueues the
 * build and returns without waiting for anything, so a training loop never stalls its launch queue on it.
 * The layout can be passed to the attention calls at once (they are ordered behind the build on the same
 * stream).  What the device finds out is looked at later: HDT_ERR_HIERARCHY (invalid ids) or HDT_ERR_SHAPE
 * (more list entries needed than the layout has room for) is returned by hdt_layout_status, which waits
 * for the build kernel, by hdt_layout_info / hdt_layout_sample_info / hdt_layout_export, and by every
 * attention call made after the report has arrived; attention calls made before that run on the lists as
 * far as they were written (always inside the layout's arrays) and their results are then meaningless.
 * The room is opts->capacity list entries if given (also for a call that waits: HDT_ERR_SHAPE instead of a
 * second attempt); otherwise a deferred build takes the most any document can need, batch * q_tiles *
 * k_tiles, as far as that stays within 256 MiB (n_pos up to about 32768 for one sample), and beyond
 * that what 256 MiB hold.  At most 1024 builds may be in flight per process.
 *
 * Errors: HDT_ERR_INVALID_ARG (NULL, negative sizes, edges outside HDT_EDGE_ALL), HDT_ERR_SHAPE (n_pos > 2^19),
 * HDT_ERR_UNSUPPORTED (tile shape), HDT_ERR_HIERARCHY (level outside [-1, HDT_MAX_LEVELS),
 * parent outside [-1, n_pos), parent[i] == i, a pad with a parent, a parent that is a pad),
 * HDT_ERR_OOM, HDT_ERR_HIP.  On error *out is NULL.
 */
hdt_status_t hdt_build_layout(const int32_t *d_level, const int32_t *d_parent, int32_t batch, int32_t n_pos,
                              const hdt_layout_opts_t *opts, void *stream, hdt_layout_t **out);

/*
 * hdt_build_cross_layout -- schedule of decoder cross-attention over a subset of the encoder's positions.
 * (Sec. 4.2, the summarisation study: the decoder of the encoder-decoder model cross-attends only to the
 * [SEC] anchors, or additionally to the [SENT] anchors, or additionally to the regular tokens.)
 *
 *   d_level_enc [batch][n_enc] int32, device: hierarchy level of each encoder position (HDT_LEVEL_PAD for pads)
 *   n_dec       decoder rows per sample
 *   level_mask  bit l set <=> encoder positions of level l are visible (e.g. 1<<1 for [SEC] only,
 *               (1<<1)|(1<<2) with [SENT], |(1<<3) with the tokens; whether [DOC], level 0, joins is the
 *               caller's choice); pads and levels outside [0, 32) are never visible
 *   opts        host, may be NULL; only tile_m / tile_n are honoured, any other option set is UNSUPPORTED
 *
 * Every decoder row attends to every visible position of its sample.  The layout is then used with the
 * ordinary attention calls, whose tensors take two lengths: q, o, d_o, dq are [batch][heads][n_dec][d] and
 * lse [batch][heads][n_dec]; k, v, dk, dv are [batch][heads][n_enc][d].  In the forward, K and V rows of the
 * visible positions are gathered by the attention kernel itself (no compacted copy is made); dk and dv of
 * invisible positions are written as zeros; a sample without visible positions gives O = 0, LSE = -inf.
 * hdt_layout_info reports n_pos = n_dec and n_kv = n_enc.  The layout holds a second schedule for the
 * backward pass (rows = encoder positions), reachable through hdt_layout_transposed.
 * When at most a quarter of the encoder's positions are visible in every sample, the layout also holds a pair
 * of schedules over the visible positions alone, and hdt_attn_bwd works on compact copies of K, V, dK, dV of
 * compact_rows (hdt_layout_info) rows per sample, which it keeps in its workspace
 * (hdt_attn_bwd_workspace_bytes grows by those four tensors): its dK/dV pass then tiles the visible rows
 * instead of all encoder rows.  Results and arguments are the same either way.
 *
 * Kernels are enqueued on `stream`; the call waits for the first of them once (it reads the number of visible
 * positions back); device memory as for hdt_build_layout, sized for the case that every position is visible.
 * batch == 0 gives an empty layout on which the attention calls are no-ops.
 * Errors: HDT_ERR_INVALID_ARG (NULL, negative sizes), HDT_ERR_SHAPE (a length of 0 or > 2^19, too many
 * entries), HDT_ERR_UNSUPPORTED (tile shape, other options), HDT_ERR_OOM, HDT_ERR_HIP.  On error *out is NULL.
 */
hdt_status_t hdt_build_cross_layout(const int32_t *d_level_enc, int32_t batch, int32_t n_enc, int32_t n_dec,
                                    uint32_t level_mask, const hdt_layout_opts_t *opts, void *stream,
                                    hdt_layout_t **out);

/* The schedule of the transposed mask that a layout holds for the backward pass (directed masks of
 * hdt_build_layout, every cross-attention layout), as a borrowed handle for hdt_layout_info /
 * hdt_layout_sample_info / hdt_layout_export: *out is NULL if the layout has none (symmetric mask); it is
 * owned by `layout` and dies with it. */
hdt_status_t hdt_layout_transposed(const hdt_layout_t *layout, const hdt_layout_t **out);

/* The outcome of a deferred build (opts->deferred): waits until the build kernel has reported (not for the
 * stream), then returns HDT_OK, HDT_ERR_HIERARCHY or HDT_ERR_SHAPE as hdt_build_layout would have.
 * *h_entries_needed (may be NULL) receives the number of list entries the schedule needs, which is what
 * opts->capacity must be at least for the build to succeed.  On a layout built without `deferred` it returns
 * HDT_OK at once. */
hdt_status_t hdt_layout_status(const hdt_layout_t *layout, int64_t *h_entries_needed);

/* Sizes of a layout (host struct).  n_tiles and nnz are read back from the device by the first call
 * of hdt_layout_info / hdt_layout_sample_info / hdt_layout_export on a layout, which synchronises
 * the device; later calls are host-only. */
hdt_status_t hdt_layout_info(const hdt_layout_t *layout, hdt_layout_info_t *h_info);

/* Surviving tiles and allowed pairs of one sample. */
hdt_status_t hdt_layout_sample_info(const hdt_layout_t *layout, int32_t sample, int64_t *h_n_tiles,
                                    int64_t *h_nnz);

/*
 * hdt_layout_export -- copy one sample's schedule to host arrays (for inspection and tests).
 * Any output pointer may be NULL.  Sizes, with T = the sample's n_tiles:
 *   h_kperm    int32  [n_pos]        key order: sorted slot -> position
 *   h_q_rowptr int32  [q_tiles + 1]  tiles of query tile I are entries [q_rowptr[I], q_rowptr[I+1])
 *   h_q_cols   int32  [T]            windowed: key window J of each entry, ascending inside a query tile;
 *                                    otherwise the ordinal of the entry inside its query tile
 *   h_q_keys   int32  [T][tile_n]    document position behind every key slot of every entry; -1 where the
 *                                    slot holds no key (the tail of a key list; in a windowed layout also pads,
 *                                    slots past n_pos and keys that no row of the query tile may attend to)
 *   h_q_sub    uint32 [T]            32x32 sub-block (r, c) -> bit r*(tile_n/32)+c: bits 0..15 set iff the
 *                                    sub-block is computed, i.e. holds an allowed pair (force_dense: every
 *                                    sub-block of the tile), bits 16..31 iff all its pairs are allowed
 *   h_bits     uint32 [T][tile_m][tile_n/32]  bitmap, word r*(tile_n/32)+c/32, bit c%32 <=> row r, slot c allowed
 *   h_k_colptr int32  [k_tiles + 1]  windowed layouts only: the transpose, entries of key window J
 *   h_k_rows   int32  [T]            query tile of each transposed entry, ascending inside a key window
 *   h_k_tile   int32  [T]            index (into the q-ordered entries) of each transposed entry
 * `tile_capacity` is the number of entries the T-sized arrays can hold; HDT_ERR_SHAPE if too small;
 * HDT_ERR_UNSUPPORTED if one of the h_k_* arrays is asked of a layout that is not windowed.
 * Synchronises the device.
 */
hdt_status_t hdt_layout_export(const hdt_layout_t *layout, int32_t sample, int32_t *h_kperm,
                               int32_t *h_q_rowptr, int32_t *h_q_cols, int32_t *h_q_keys, uint32_t *h_q_sub,
                               uint32_t *h_bits, int32_t *h_k_colptr, int32_t *h_k_rows, int32_t *h_k_tile,
                               int64_t tile_capacity);

/* Destroys the layout.  NULL is accepted, and the call does not wait: attention calls that use the layout may
 * still be queued or running.  Its device buffers go to a cache (at most 16 buffers / 1 GiB per process) that
 * later hdt_build_layout calls draw from; a build that takes them orders itself behind everything enqueued so far
 * on the streams this layout was built and used on (an event per other stream, nothing for its own stream, no
 * host wait).  The streams of those calls must still exist then, or the build waits for the device instead. */
hdt_status_t hdt_layout_destroy(hdt_layout_t *layout);

/* The same for a caller that has waited for the layout's build and for every call that used it (an event of its
 * own, a stream or device synchronisation): the buffers go to the cache with nothing left to wait for.  What the
 * plain call costs when layouts are built on one stream and used on another is an event recorded on the stream
 * of the attention calls, a few microseconds of that stream's time per destroyed layout. */
hdt_status_t hdt_layout_destroy_completed(hdt_layout_t *layout);

/* Returns the cached device buffers to the driver (hipFree). */
hdt_status_t hdt_release_cached_memory(void);

/*
 * hdt_attn_fwd -- forward pass over the surviving tiles (App. A.1, Alg. 1: per query tile, loop
 * over its key tiles, gathered row by row through the layout's key positions, mask, online softmax,
 * accumulate P V; O and the softmax statistics are
 * written once at the end instead of once per key tile).
 *
 *   q, k, v  device, [batch][heads][n_pos][head_dim], dtype `dt`
 *   o        device, same shape and dtype: O = softmax(mask(Q K^T * softmax_scale)) V; 0 on pad rows
 *   lse      device, [batch][heads][n_pos] float: natural-log sum of exp of the masked, scaled logits
 *            of each row; -inf on pad rows
 *   head_dim 64 or 128;  softmax_scale > 0 (the paper uses 1/sqrt(head_dim))
 *
 * HDT_BF16 needs a layout with tiles 128 x 64 or 64 x 32 (the backward pass is the faster one on 64 x 32 tiles,
 * by more than their build costs, and so is the forward at head size 128; a layout used for the forward only at
 * head size 64 is best left at the default); HDT_F32 takes any layout.  batch and n_pos come from the layout.  Errors: INVALID_ARG, UNSUPPORTED (head_dim, dtype, tile shape), HDT_ERR_HIP (launch).
 */
hdt_status_t hdt_attn_fwd(const hdt_layout_t *layout, const void *q, const void *k, const void *v, void *o,
                          float *lse, int32_t heads, int32_t head_dim, hdt_dtype_t dt, float softmax_scale,
                          void *stream);

/*
 * hdt_attn_fwd_ws -- hdt_attn_fwd with a workspace.  Where a few row tiles would each walk a very long key list
 * (a cross-attention layout with the regular tokens visible: Sec. 4.2, the widest setting of the summarisation
 * study), the lists are cut into pieces that separate workgroups walk, each producing a partial O and LSE in the
 * workspace, and a small kernel combines them (O = sum_p exp(LSE_p - LSE) O_p, LSE = log sum_p exp(LSE_p); a fixed
 * order, so the result is reproducible).  Results agree with hdt_attn_fwd within the rounding of the partial O to
 * bf16.  hdt_attn_fwd_workspace_bytes says how much room that takes for a layout, head count and head size: 0
 * means hdt_attn_fwd_ws does what hdt_attn_fwd does (every self-attention layout, HDT_F32, short lists); with
 * less room than that (or NULL) it also does.  `workspace`: device, 16-byte aligned, scratch only.
 */
size_t hdt_attn_fwd_workspace_bytes(const hdt_layout_t *layout, int32_t heads, int32_t head_dim, hdt_dtype_t dt);
hdt_status_t hdt_attn_fwd_ws(const hdt_layout_t *layout, const void *q, const void *k, const void *v, void *o,
                             float *lse, int32_t heads, int32_t head_dim, hdt_dtype_t dt, float softmax_scale,
                             void *workspace, size_t workspace_bytes, void *stream);

/* Bytes of device workspace hdt_attn_bwd needs (0 on bad arguments). */
size_t hdt_attn_bwd_workspace_bytes(const hdt_layout_t *layout, int32_t heads, int32_t head_dim,
                                    hdt_dtype_t dt);

/*
 * hdt_attn_bwd -- gradients of the forward pass (the paper gives no backward; this is the
 * gradient of the definition in Sec. 3.2, evaluated over the same surviving tiles):
 *   D_i = sum_c dO_ic O_ic,  P = exp(S - LSE),  dV = P^T dO,  dP = dO V^T,  dS = P o (dP - D),
 *   dQ = scale dS K,  dK = scale dS^T Q.
 *
 *   q, k, v, o, d_o   device, [batch][heads][n_pos][head_dim], dtype `dt` (o, lse from hdt_attn_fwd)
 *   lse               device, [batch][heads][n_pos] float
 *   dq, dk, dv        device, outputs, same shape and dtype; rows of pad positions are written as 0
 *   workspace         device, at least hdt_attn_bwd_workspace_bytes() bytes, 16-byte aligned; scratch only
 */
hdt_status_t hdt_attn_bwd(const hdt_layout_t *layout, const void *q, const void *k, const void *v,
                          const void *o, const float *lse, const void *d_o, void *dq, void *dk, void *dv,
                          int32_t heads, int32_t head_dim, hdt_dtype_t dt, float softmax_scale,
                          void *workspace, size_t workspace_bytes, void *stream);

/*
 * hdt_attn_bwd_no_alloc -- hdt_attn_bwd for callers that cannot allocate device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same computation with the same arguments
 * except the workspace, which is an array inside the library (HDT_NO_ALLOC_WORKSPACE_BYTES of device memory
 * that every GPU the library runs on holds until the process ends).  The call allocates nothing and frees
 * nothing.  HDT_ERR_SHAPE if hdt_attn_bwd_workspace_bytes() of the call exceeds the array (for a self-attention
 * layout: batch * heads * n_pos > 2^20, two floats each); the other errors are hdt_attn_bwd's.  All calls on one GPU share the
 * array: calls that may overlap there (different streams, different host threads) race; calls on one stream
 * do not.  Nothing in the array has to survive between calls and nothing in it has to start at zero.
 */
#define HDT_NO_ALLOC_WORKSPACE_BYTES (8u << 20)
hdt_status_t hdt_attn_bwd_no_alloc(const hdt_layout_t *layout, const void *q, const void *k, const void *v,
                                   const void *o, const float *lse, const void *d_o, void *dq, void *dk, void *dv,
                                   int32_t heads, int32_t head_dim, hdt_dtype_t dt, float softmax_scale,
                                   void *stream);

/*
 * Hierarchical positional encoding (Sec. 3.2 "Hierarchical Positional Encoding", Eq. pos_enc, Fig. 3):
 * every position carries one linear index p^l per hierarchy level l = 1 .. n_levels (level 0 needs none);
 *     HPE(p, c) = sum_l sin(w_k p^l) if c = 2k,  sum_l cos(w_k p^l) if c = 2k + 1,  w_k = 10000^(-2k/d_model),
 * is added to the embeddings.
 *
 * hdt_parents_from_levels -- d_level [batch][n_pos] int32 (device) -> d_parent [batch][n_pos] int32 (device) for
 *   documents in the layout of Sec. 3.2 (every anchor in front of what it summarises, i.e. pre-order): the
 *   parent of a position of level l > 0 is the nearest earlier position of level l - 1; level 0, pads, levels
 *   outside [0, HDT_MAX_LEVELS) and positions without such a predecessor get -1.  The front end for callers
 *   that only know where sections and sentences start.
 * hdt_index_vectors -- level/parent ids (as for hdt_build_layout) -> d_p [batch][n_pos][n_levels] int32,
 *   device: entry l-1 of position i = the 1-based ordinal, among the children of its parent in document
 *   order, of i's ancestor-or-self whose level is l; 0 if there is none ([DOC] = (0,0,0), k-th [SEC] =
 *   (k,0,0), its m-th [SENT] = (k,m,0), that sentence's t-th token = (k,m,t)); pads carry zeros.
 *   `workspace`: device scratch of hdt_index_vectors_workspace_bytes(batch, n_pos) bytes, 16-byte aligned.
 *   The ids are not validated here (hdt_build_layout does that); out-of-range parents count as roots.
 * hdt_hpe_table -- d_table [rows][d_model] float, device: T[v][c] = sin / cos (w_k v); d_model % 8 == 0.
 * hdt_hpe_add -- x [batch][n_pos][d_model] (dtype dt, device, in place): x += sum_l T[p^l]; indices outside
 *   [0, table_rows) are evaluated directly, so any table size (even 0) gives the same result.
 * All of them only enqueue work on `stream`.  Errors: INVALID_ARG, SHAPE, UNSUPPORTED (dtype), HDT_ERR_HIP.
 */
hdt_status_t hdt_parents_from_levels(const int32_t *d_level, int32_t batch, int32_t n_pos, int32_t *d_parent,
                                     void *stream);
size_t hdt_index_vectors_workspace_bytes(int32_t batch, int32_t n_pos);
hdt_status_t hdt_index_vectors(const int32_t *d_level, const int32_t *d_parent, int32_t batch, int32_t n_pos,
                               int32_t n_levels, int32_t *d_p, void *workspace, size_t workspace_bytes,
                               void *stream);
hdt_status_t hdt_hpe_table(float *d_table, int32_t rows, int32_t d_model, void *stream);
hdt_status_t hdt_hpe_add(const int32_t *d_p, int32_t batch, int32_t n_pos, int32_t n_levels, const float *d_table,
                         int32_t table_rows, void *x, int32_t d_model, hdt_dtype_t dt, void *stream);

/* Text of a status code / of the last error on this thread (never NULL). */
const char *hdt_status_string(hdt_status_t status);
const char *hdt_last_error(void);

/*
 * Per-kernel timing for benchmarks.  With timing enabled every kernel launch of the library is
 * bracketed by HIP events on the stream it is launched on.  hdt_timing_read synchronises those
 * events and returns, for up to `capacity` kernels, the kernel name (pointer to a static string),
 * the number of launches and the summed duration in milliseconds since the last hdt_timing_reset;
 * it returns the number of distinct kernels seen.  Not thread-safe; meant for single-threaded
 * benchmark loops.
 */
hdt_status_t hdt_timing_enable(int32_t enable);
hdt_status_t hdt_timing_reset(void);
int32_t hdt_timing_read(const char **h_names, int64_t *h_launches, double *h_total_ms, int32_t capacity);

/*
 * A measuring stick for benchmarks (no part of the attention path): enqueues a kernel of `workgroups`
 * workgroups of four waves that does nothing but `iters` x 32 bf16 contraction instructions per wave (the
 * 32 x 32 x 16 form the attention kernels use, four independent accumulator chains), and returns in *h_flop the
 * floating-point operations that launch performs.  Timed by the caller (events on `stream`), it gives the MFMA
 * rate the chip sustains at the clock it holds under that load.  d_sink: device, 4 bytes, never written.
 * Errors: INVALID_ARG, HDT_ERR_HIP.
 */
hdt_status_t hdt_probe_mfma_bf16(int32_t workgroups, int32_t iters, float *d_sink, double *h_flop, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* HDT_H */
