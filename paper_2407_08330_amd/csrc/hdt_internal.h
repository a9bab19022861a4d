// Internal declarations shared by the translation units of libhdt (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <memory>
#include <stdint.h>

#include <string>
#include <vector>

#include "hdt.h"

#define HDT_LAYOUT_MAGIC 0x4844544cu  // "HDTL"

// Device-side view of a tile schedule, passed by value to the attention kernels.
//
// Every query tile (b, I) owns a contiguous run of list entries; an entry is one key tile: bn key
// slots, each naming the document position to gather (q_keys, negative = no key), with the bitmaps of the
// allowed pairs.  Windowed layouts fill an entry's slots from a window of the key order kperm, the
// default layouts with the next bn keys of the query tile's own key list; the kernels do not care.
// In a windowed layout an entry may turn out to hold no allowed pair (only for documents that are not
// in pre-order); it keeps its place with an all-zero summary (q_sub == 0) and all-zero bitmaps, which
// makes every kernel skip it, and hdt_layout_export filters it out.
struct HdtSchedule {
    int32_t batch, n_pos;  // n_pos: rows per sample of the row-side tensors (the ones tiled by bm)
    int32_t n_kv;          // rows per sample of the gathered tensors (= n_pos for self-attention)
    // A schedule whose key lists are cut into several pieces (hdt_cross.hip) lists every row tile once per piece:
    // row tile I works on the rows of tile I % tr_own of the row-side INPUT tensors, which have n_own rows per
    // sample, and writes its (partial) results as rows of tile I of tensors with n_pos rows.  Otherwise
    // tr_own == tr and n_own == n_pos.
    int32_t n_own, tr_own;
    int32_t bm, bn;        // tile shape (query rows x key slots)
    int32_t tr, tc;        // tiles per sample along queries / keys
    int32_t n_slots;       // tc * bn: length of one sample's padded key order
    int32_t wpr;           // bitmap words per tile row = bn / 32
    const int32_t *kperm;  // [batch][n_slots] sorted slot -> position, -1 beyond n_pos (not read by the attention kernels)
    const int32_t *q_range;   // [batch][tr][2] first and one-past-last list entry of query tile (b, I)
    const int32_t *q_cols;    // [entries] windowed layouts: key window of each entry
    // [entries][bn] document position behind each key slot; a slot without a key (no key left, a pad, a key
    // no row of the tile may attend to) holds ~f < 0, f being the first real row of the tile: the row the
    // attention kernels gather in its place (see gather_row in hdt_tile.h)
    const int32_t *q_keys;
    const uint32_t *q_sub;    // [entries] 32x32 sub-block summary (bits 0..15 any, 16..31 all)
    // [entries][(bm/32)*(bn/32)][16] per 32x32 sub-block (r, c) = index r*(bn/32)+c: bit l of word e <=>
    // row 32r + l%32, column 32c + (l/32)*4 + 8*(e/4) + e%4 allowed: the lane mask of MFMA accumulator register e
    const unsigned long long *bits_rm;
    // [batch][n_pos] >= 0 iff the row is a real position (may attend to anything), or NULL = every row is:
    // the level ids of a self-attention layout, the ranks of a cross-attention layout's encoder rows
    const int32_t *row_flag;
};

// whether row r of list entry t may attend to the key in slot c (plain indexing of bits_rm)
__host__ __device__ inline bool hdt_pair_allowed(const unsigned long long *bits_rm, int bm, int wpr, size_t t, int r, int c)
{
    const size_t sb = (size_t)(r >> 5) * wpr + (c >> 5), nsub = (size_t)(bm >> 5) * wpr;
    const int l = (r & 31) + 32 * ((c >> 2) & 1), e = ((c & 31) >> 3) * 4 + (c & 3);
    return (bits_rm[(t * nsub + sb) * 16 + e] >> l) & 1ull;
}

// The streams on which work that touches a layout's buffers has been enqueued (its build, the attention calls):
// what a later owner of those buffers orders itself after.
struct HdtStreams {
    static constexpr int kMax = 4;
    hipStream_t s[kMax] = {};
    int n = 0;
    bool more = false;  // more than kMax streams: the later owner waits for the whole device instead
    void add(hipStream_t x)
    {
        for (int i = 0; i < n; i++)
            if (s[i] == x) return;
        if (n < kMax)
            s[n++] = x;
        else
            more = true;
    }
};

struct hdt_layout {
    uint32_t magic;
    mutable HdtStreams streams;  // of the handle the caller holds; the layouts it owns are used through it
    HdtSchedule s;       // pointers into the arenas
    int32_t device;      // device the buffers live on
    int32_t force_dense; // every candidate counts as a tile, empty or not
    int32_t windowed;    // key tiles are windows of the key order (else per-query-tile key lists)
    int32_t edges;       // OR of HDT_EDGE_*
    int32_t cross;       // 1: a cross-attention layout (rows and gathered tensors differ; hdt_cross.hip)
    uint32_t cross_level_mask;
    // directed masks (edges without up/down symmetry): the schedule of the transposed mask (rows = keys,
    // list entries = the queries attending to them), owned by this layout; NULL for symmetric masks
    hdt_layout *transposed;
    // Cross-attention layouts with few visible positions (hdt_cross.hip): a second pair of schedules in the index
    // space of the visible positions (a position's row = its rank among them), on which the backward runs with
    // compact copies of K and V.  `compact` schedules the dQ pass (keys = ranks), compact->transposed the
    // dK/dV pass (rows = ranks); all owned by this layout.  NULL: no such pair.
    hdt_layout *compact;
    const int32_t *cross_sel;    // [batch][n_kv] visible positions in document order (device)
    const int32_t *cross_count;  // [batch] their number (device)
    const int32_t *cross_rank;   // [batch][n_kv] rank among the visible positions, -1 = not visible (device)
    int32_t n_compact;           // rows per (sample, head) of the compact tensors
    // Long key lists cut into 2, 4 or 8 pieces (hdt_cross.hip): the entry ranges of the row tiles of every piece,
    // [batch][pieces * tr][2] each (device, in this layout's first arena); NULL if the lists are short
    const int32_t *cross_split_range[3];
    int32_t cross_entries_max;   // entries of the longest key list (host copy)
    int64_t capacity;    // entries the per-tile arrays can hold
    int64_t device_bytes;
    void *arena;         // key order, list pointers, scratch of the build
    void *arena2;        // per-tile arrays
    size_t arena_bytes, arena2_bytes;
    const int32_t *d_cnt;          // [entries] allowed pairs of each entry (device)
    const int32_t *d_row;          // [entries] query tile (global numbering b * tr + I) of each entry (device)
    mutable int64_t n_entries;     // list entries of all samples (a deferred build: once its report has been read)
    // [batch][2] = (surviving tiles, allowed pairs) per sample; read back from the device by the first
    // query that needs them (hdt_layout_stats), not by the build
    mutable std::vector<int64_t> h_stats;
    mutable bool stats_ready;
    // Key-list layouts do not need the global key order; it is sorted from the layout's copy of the ids
    // on demand (hdt_layout_ensure_kperm).
    mutable bool kperm_ready;
    int32_t no_sort;
    int32_t *sort_hist, *sort_counters;
    const int32_t *level_copy, *parent_copy;
    // A deferred build (hdt_layout_opts_t.deferred) has not looked at the device's report yet: whether the
    // hierarchy was valid and how many list entries it needed.  hdt_layout_resolve reads it (once).
    mutable bool pending;
    mutable hdt_status_t build_status;     // what the report said, once it has been read
    mutable int64_t entries_needed;        // list entries the build needed (-1: not known yet)
    mutable char build_error[320];         // text of build_status
    const unsigned long long *report;      // the build's word of pinned host memory
    const unsigned long long *report_dev;  // the same word in the layout's own device memory
    uint32_t ticket, ticket_before;        // the build's ticket; the one its report slot held when it was enqueued
};

// --- error reporting (hdt_api.hip) ---
hdt_status_t hdt_fail(hdt_status_t st, const char *fmt, ...);
#define HDT_HIP_TRY(expr)                                                                     \
    do {                                                                                      \
        hipError_t _e = (expr);                                                               \
        if (_e != hipSuccess)                                                                 \
            return hdt_fail(_e == hipErrorOutOfMemory ? HDT_ERR_OOM : HDT_ERR_HIP, "%s: %s", \
                            #expr, hipGetErrorString(_e));                                    \
    } while (0)

bool hdt_layout_ok(const hdt_layout_t *l);
// Reads the report of a deferred build: with `wait` it returns once the report is in (it waits for the build
// kernel, not for the stream), without it only looks.  Returns the build's status as far as it is known (HDT_OK
// while nothing is known); covers the transposed schedule a directed mask brings.  (hdt_layout.hip)
hdt_status_t hdt_layout_resolve(const hdt_layout_t *l, bool wait);
hdt_status_t hdt_layout_ensure_kperm(const hdt_layout_t *l);  // sorts s.kperm if the build did not (waits for the device) (hdt_layout.hip)
hdt_status_t hdt_layout_stats(const hdt_layout_t *l);  // fills h_stats once (waits for the device) (hdt_layout.hip)
// What the next owner of a released buffer has to wait for.  A stream on which layouts are also built is only
// remembered (`lazy`): the next build is most likely enqueued there too and needs nothing; should it come on another
// stream, an event recorded then covers the work in question (and whatever was enqueued since).  For any other
// stream an event is recorded at the release, so that a build on a second stream waits for exactly the calls that
// used the buffer and not for the ones enqueued later.
struct HdtFence {
    hipEvent_t ev;
    hipStream_t stream;
    ~HdtFence();  // returns the event to a free list (hdt_layout.hip)
};
struct HdtUsers {
    HdtStreams lazy;
    std::vector<std::shared_ptr<HdtFence>> fences;
    bool whole_device = false;
};
HdtUsers hdt_users_at_release(const HdtStreams &streams);  // records the events
void hdt_note_build_stream(hipStream_t st);                  // a layout build is being enqueued on `st`
// hands the device buffers back to the cache (hdt_layout.hip)
void hdt_layout_release(hdt_layout_t *l, const HdtUsers &users);
void hdt_layout_note_stream(const hdt_layout_t *l, hipStream_t st);  // an attention call is about to use `l` on `st`
HdtStreams hdt_layout_streams(const hdt_layout_t *l);
// device buffer from the cache of destroyed layouts' buffers, or a new one; *got = its real size (hdt_layout.hip)
// `next_user`: the stream on which the buffer's new owner enqueues its work
hipError_t hdt_pool_alloc(void **out, size_t bytes, size_t *got, hipStream_t next_user);

// --- key lists of a cross-attention layout cut into pieces that separate workgroups walk (hdt_cross.hip) ---
int hdt_cross_pieces(const hdt_layout_t *l, int heads);  // 1, 2, 4 or 8 for this many heads
size_t hdt_cross_fwd_workspace_bytes(const hdt_layout_t *l, int heads, int head_dim);
size_t hdt_cross_dq_workspace_bytes(const hdt_layout_t *l, int heads, int head_dim);
hdt_status_t hdt_cross_fwd_split(const hdt_layout_t *l, const void *q, const void *k, const void *v, void *o, float *lse,
                                 int heads, int head_dim, float scale, void *workspace, hipStream_t st);
hdt_status_t hdt_cross_bwd_split(const hdt_layout_t *l, const void *q, const void *k, const void *v, const void *o,
                                 const float *lse, const void *d_o, void *dq, void *dk, void *dv, int heads,
                                 int head_dim, float scale, void *workspace, hipStream_t st);

// --- backward of a cross-attention layout with a compact pair (hdt_cross.hip) ---
size_t hdt_cross_compact_workspace_bytes(const hdt_layout_t *l, int heads, int head_dim, int elem_bytes);
hdt_status_t hdt_cross_bwd_compact(const hdt_layout_t *l, const void *q, const void *k, const void *v, const void *o,
                                   const float *lse, const void *d_o, void *dq, void *dk, void *dv, int heads,
                                   int head_dim, bool bf16, float scale, void *workspace, hipStream_t st);

// --- per-kernel timing (hdt_api.hip) ---
struct HdtTimer {  // brackets one kernel launch with events when timing is enabled
    HdtTimer(const char *name, hipStream_t stream);
    ~HdtTimer();
    int slot;
    hipStream_t stream;
};

// --- kernels' host launchers (each validates nothing; callers have done it) ---
hdt_status_t hdt_launch_fwd_bf16(const HdtSchedule &s, const void *q, const void *k, const void *v, void *o,
                                 float *lse, int heads, int head_dim, float scale, hipStream_t st);
hdt_status_t hdt_launch_fwd_f32(const HdtSchedule &s, const float *q, const float *k, const float *v, float *o,
                                float *lse, int heads, int head_dim, float scale, hipStream_t st);
// backward launchers: `s` schedules the dQ pass, `s_transposed` (the transposed mask's schedule; the same as `s` for
// symmetric masks) the dK/dV pass.  `delta`: room for the rows' scalars, hdt_bwd_row_scalars_bytes(batch * heads * n_pos)
// (two floats per row for the bf16 kernels: -D and -LSE / scale side by side; the fp32 kernels keep D in the first half).
inline size_t hdt_bwd_row_scalars_bytes(size_t rows) { return (2 * rows * sizeof(float) + 255) & ~(size_t)255; }
hdt_status_t hdt_launch_bwd_bf16(const HdtSchedule &s, const HdtSchedule &s_transposed, const void *q, const void *k, const void *v,
                                 const void *o, const float *lse, const void *d_o, void *dq, void *dk,
                                 void *dv, int heads, int head_dim, float scale, float *ws_delta,
                                 hipStream_t st);
hdt_status_t hdt_launch_bwd_f32(const HdtSchedule &s, const HdtSchedule &s_transposed, const float *q, const float *k, const float *v,
                                const float *o, const float *lse, const float *d_o, float *dq, float *dk,
                                float *dv, int heads, int head_dim, float scale, float *ws_delta,
                                hipStream_t st);
