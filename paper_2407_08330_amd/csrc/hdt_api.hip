// C-ABI entry points: argument checking, error text, layout lifetime and export, dispatch to the
// kernel launchers.  No arithmetic of the method lives here.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <mutex>

#include "hdt_internal.h"

// ---------------------------------------------------------------------------- errors
static thread_local char g_err[512] = "";

hdt_status_t hdt_fail(hdt_status_t st, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

extern "C" __attribute__((visibility("default"))) const char *hdt_last_error(void) { return g_err; }

extern "C" __attribute__((visibility("default"))) const char *hdt_status_string(hdt_status_t s)
{
    switch (s) {
    case HDT_OK: return "HDT_OK";
    case HDT_ERR_INVALID_ARG: return "HDT_ERR_INVALID_ARG";
    case HDT_ERR_SHAPE: return "HDT_ERR_SHAPE";
    case HDT_ERR_HIERARCHY: return "HDT_ERR_HIERARCHY";
    case HDT_ERR_UNSUPPORTED: return "HDT_ERR_UNSUPPORTED";
    case HDT_ERR_OOM: return "HDT_ERR_OOM";
    case HDT_ERR_HIP: return "HDT_ERR_HIP";
    }
    return "HDT_ERR_UNKNOWN";
}

bool hdt_layout_ok(const hdt_layout_t *l) { return l != nullptr && l->magic == HDT_LAYOUT_MAGIC; }

// ---------------------------------------------------------------------------- timing
namespace {
struct TimedLaunch {
    const char *name;
    hipEvent_t start, stop;
};
bool g_timing = false;
std::vector<TimedLaunch> g_launches;        // since the last reset
std::vector<hipEvent_t> g_event_pool;       // events free for reuse
const size_t kMaxTimedLaunches = 1 << 16;

hipEvent_t take_event()
{
    if (!g_event_pool.empty()) {
        hipEvent_t e = g_event_pool.back();
        g_event_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}
}  // namespace

HdtTimer::HdtTimer(const char *name, hipStream_t st) : slot(-1), stream(st)
{
    if (!g_timing || g_launches.size() >= kMaxTimedLaunches) return;
    TimedLaunch t{name, take_event(), take_event()};
    if (!t.start || !t.stop) return;
    (void)hipEventRecord(t.start, stream);
    slot = (int)g_launches.size();
    g_launches.push_back(t);
}

HdtTimer::~HdtTimer()
{
    if (slot >= 0) (void)hipEventRecord(g_launches[slot].stop, stream);
}

extern "C" __attribute__((visibility("default"))) hdt_status_t hdt_timing_enable(int32_t enable)
{
    g_timing = enable != 0;
    return HDT_OK;
}

extern "C" __attribute__((visibility("default"))) hdt_status_t hdt_timing_reset(void)
{
    for (auto &t : g_launches) {
        (void)hipEventSynchronize(t.stop);
        g_event_pool.push_back(t.start);
        g_event_pool.push_back(t.stop);
    }
    g_launches.clear();
    return HDT_OK;
}

extern "C" __attribute__((visibility("default"))) int32_t hdt_timing_read(const char **names, int64_t *launches, double *total_ms, int32_t capacity)
{
    std::vector<const char *> seen;
    std::vector<int64_t> cnt;
    std::vector<double> ms;
    for (auto &t : g_launches) {
        if (hipEventSynchronize(t.stop) != hipSuccess) continue;
        float dt = 0.f;
        if (hipEventElapsedTime(&dt, t.start, t.stop) != hipSuccess) continue;
        size_t i = 0;
        for (; i < seen.size(); i++)
            if (seen[i] == t.name || strcmp(seen[i], t.name) == 0) break;
        if (i == seen.size()) {
            seen.push_back(t.name);
            cnt.push_back(0);
            ms.push_back(0.0);
        }
        cnt[i] += 1;
        ms[i] += dt;
    }
    for (size_t i = 0; i < seen.size() && (int32_t)i < capacity; i++) {
        if (names) names[i] = seen[i];
        if (launches) launches[i] = cnt[i];
        if (total_ms) total_ms[i] = ms[i];
    }
    return (int32_t)seen.size();
}

// ---------------------------------------------------------------------------- layout queries
extern "C" __attribute__((visibility("default"))) hdt_status_t hdt_layout_info(const hdt_layout_t *layout, hdt_layout_info_t *info)
{
    if (!hdt_layout_ok(layout) || !info) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_layout_info: NULL or invalid layout");
    const hdt_layout_t *l = layout;
    if (hdt_status_t st = hdt_layout_stats(l)) return st;
    info->batch = l->s.batch;
    info->n_pos = l->s.n_pos;
    info->tile_m = l->s.bm;
    info->tile_n = l->s.bn;
    info->q_tiles = l->s.tr;
    info->k_tiles = l->s.tc;
    info->windowed = l->windowed;
    info->edges = l->edges;
    info->n_tiles = 0;
    info->nnz = 0;
    for (int b = 0; b < l->s.batch; b++) {
        info->n_tiles += l->h_stats[2 * b];
        info->nnz += l->h_stats[2 * b + 1];
    }
    info->device_bytes = l->device_bytes;
    info->n_kv = l->s.n_kv;
    info->cross = l->cross;
    info->cross_level_mask = l->cross_level_mask;
    info->compact_rows = l->compact ? l->n_compact : 0;
    return HDT_OK;
}

extern "C" __attribute__((visibility("default"))) hdt_status_t hdt_layout_status(const hdt_layout_t *layout,
                                                                                  int64_t *entries_needed)
{
    if (!hdt_layout_ok(layout)) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_layout_status: NULL or invalid layout");
    const hdt_status_t st = hdt_layout_resolve(layout, true);
    if (entries_needed) {
        *entries_needed = layout->entries_needed;
        if (layout->transposed && layout->transposed->entries_needed > *entries_needed)
            *entries_needed = layout->transposed->entries_needed;
    }
    return st;
}

extern "C" __attribute__((visibility("default"))) hdt_status_t hdt_layout_sample_info(const hdt_layout_t *layout, int32_t sample, int64_t *n_tiles,
                                               int64_t *nnz)
{
    if (!hdt_layout_ok(layout)) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_layout_sample_info: invalid layout");
    if (sample < 0 || sample >= layout->s.batch)
        return hdt_fail(HDT_ERR_SHAPE, "hdt_layout_sample_info: sample %d outside [0, %d)", sample, layout->s.batch);
    const hdt_layout_t *l = layout;
    if (hdt_status_t st = hdt_layout_stats(l)) return st;
    if (n_tiles) *n_tiles = l->h_stats[2 * sample];
    if (nnz) *nnz = l->h_stats[2 * sample + 1];
    return HDT_OK;
}

extern "C" __attribute__((visibility("default"))) hdt_status_t hdt_layout_export(
    const hdt_layout_t *layout, int32_t sample, int32_t *kperm, int32_t *q_rowptr, int32_t *q_cols, int32_t *q_keys,
    uint32_t *q_sub, uint32_t *bits, int32_t *k_colptr, int32_t *k_rows, int32_t *k_tile, int64_t tile_capacity)
{
    if (!hdt_layout_ok(layout)) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_layout_export: invalid layout");
    const HdtSchedule &s = layout->s;
    if (sample < 0 || sample >= s.batch)
        return hdt_fail(HDT_ERR_SHAPE, "hdt_layout_export: sample %d outside [0, %d)", sample, s.batch);
    if (hdt_status_t st = hdt_layout_stats(layout)) return st;
    const int64_t T = layout->h_stats[2 * (size_t)sample];
    if (kperm && layout->cross)
        return hdt_fail(HDT_ERR_UNSUPPORTED, "hdt_layout_export: a cross-attention layout has no key order");
    if ((k_colptr || k_rows || k_tile) && !layout->windowed)
        return hdt_fail(HDT_ERR_UNSUPPORTED, "hdt_layout_export: only a windowed layout has a transpose by key window");
    const bool want_tiles = q_cols || q_keys || q_sub || bits || k_rows || k_tile;
    if (want_tiles && tile_capacity < T)
        return hdt_fail(HDT_ERR_SHAPE, "hdt_layout_export: capacity %lld < %lld tiles", (long long)tile_capacity,
                        (long long)T);
    HDT_HIP_TRY(hipDeviceSynchronize());
    if (kperm && s.n_pos > 0)
        if (hdt_status_t st = hdt_layout_ensure_kperm(layout)) return st;
    if (kperm && s.n_pos > 0)
        HDT_HIP_TRY(hipMemcpy(kperm, s.kperm + (size_t)sample * s.n_slots, sizeof(int32_t) * s.n_pos,
                              hipMemcpyDeviceToHost));
    // the device lists hold every candidate tile; the exported schedule keeps those with an allowed pair
    // (all of them for a dense layout) and is numbered from 0
    std::vector<int32_t> rg((size_t)s.tr * 2, 0);
    if (s.tr > 0)
        HDT_HIP_TRY(hipMemcpy(rg.data(), s.q_range + (size_t)sample * s.tr * 2, sizeof(int32_t) * s.tr * 2,
                              hipMemcpyDeviceToHost));
    const int64_t E = layout->n_entries;  // entries of all samples (a query tile's entries are contiguous)
    std::vector<int32_t> cols((size_t)E), cnt((size_t)E);
    std::vector<uint32_t> sub((size_t)E);
    if (E > 0) {
        if (layout->windowed)
            HDT_HIP_TRY(hipMemcpy(cols.data(), s.q_cols, sizeof(int32_t) * E, hipMemcpyDeviceToHost));
        HDT_HIP_TRY(hipMemcpy(cnt.data(), layout->d_cnt, sizeof(int32_t) * E, hipMemcpyDeviceToHost));
        HDT_HIP_TRY(hipMemcpy(sub.data(), s.q_sub, sizeof(uint32_t) * E, hipMemcpyDeviceToHost));
    }
    std::vector<int32_t> new_rp((size_t)s.tr + 1, 0), keep_col, keep_row, keep_entry;
    for (int I = 0; I < s.tr; I++) {
        if (rg[2 * I] < 0 || rg[2 * I + 1] < rg[2 * I] || rg[2 * I + 1] > E)
            return hdt_fail(HDT_ERR_HIP, "hdt_layout_export: corrupt list range of query tile %d", I);
        for (int32_t e = rg[2 * I]; e < rg[2 * I + 1]; e++)
            if (cnt[e] > 0 || layout->force_dense) {
                keep_col.push_back(layout->windowed ? cols[e] : e - rg[2 * I]);
                keep_row.push_back(I);
                keep_entry.push_back(e);
            }
        new_rp[I + 1] = (int32_t)keep_col.size();
    }
    if ((int64_t)keep_col.size() != T)
        return hdt_fail(HDT_ERR_HIP, "hdt_layout_export: inconsistent tile counts (%zu listed, %lld counted)",
                        keep_col.size(), (long long)T);
    if (q_rowptr) memcpy(q_rowptr, new_rp.data(), sizeof(int32_t) * (s.tr + 1));
    const size_t words = (size_t)s.bm * s.wpr;
    std::vector<unsigned long long> rm((size_t)(s.bm / 32) * s.wpr * 16);
    for (int64_t t = 0; t < T; t++) {
        if (q_cols) q_cols[t] = keep_col[t];
        if (q_sub) q_sub[t] = sub[keep_entry[t]];
        if (q_keys) {  // slots without a key: the device keeps the row gathered in their place, complemented
            HDT_HIP_TRY(hipMemcpy(q_keys + (size_t)t * s.bn, s.q_keys + (size_t)keep_entry[t] * s.bn,
                                  sizeof(int32_t) * s.bn, hipMemcpyDeviceToHost));
            for (int c = 0; c < s.bn; c++)
                if (q_keys[(size_t)t * s.bn + c] < 0) q_keys[(size_t)t * s.bn + c] = -1;
        }
        if (bits) {  // row-major bitmaps are derived here from the lane masks the device keeps
            HDT_HIP_TRY(hipMemcpy(rm.data(), s.bits_rm + (size_t)keep_entry[t] * rm.size(),
                                  sizeof(unsigned long long) * rm.size(), hipMemcpyDeviceToHost));
            uint32_t *out = bits + (size_t)t * words;
            memset(out, 0, sizeof(uint32_t) * words);
            for (int r = 0; r < s.bm; r++)
                for (int c = 0; c < s.bn; c++)
                    if (hdt_pair_allowed(rm.data(), s.bm, s.wpr, 0, r, c)) out[(size_t)r * s.wpr + (c >> 5)] |= 1u << (c & 31);
        }
    }
    // transpose by key tile (query tiles ascending): the kernels do not need it (the mask is symmetric,
    // so the backward walks the same lists); it is derived here for callers that want both views
    if (k_colptr || k_rows || k_tile) {
        std::vector<int32_t> cp((size_t)s.tc + 1, 0);
        for (int64_t t = 0; t < T; t++) cp[keep_col[t] + 1]++;
        for (int J = 0; J < s.tc; J++) cp[J + 1] += cp[J];
        if (k_colptr) memcpy(k_colptr, cp.data(), sizeof(int32_t) * (s.tc + 1));
        std::vector<int32_t> cur(cp.begin(), cp.end() - 1);
        for (int64_t t = 0; t < T; t++) {  // t ascends with the query tile, so rows come out ascending
            const int32_t e = cur[keep_col[t]]++;
            if (k_rows) k_rows[e] = keep_row[t];
            if (k_tile) k_tile[e] = (int32_t)t;
        }
    }
    return HDT_OK;
}

extern "C" __attribute__((visibility("default"))) hdt_status_t hdt_layout_transposed(const hdt_layout_t *layout,
                                                                                      const hdt_layout_t **out)
{
    if (!hdt_layout_ok(layout) || !out) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_layout_transposed: NULL or invalid layout");
    *out = layout->transposed;
    return HDT_OK;
}

static hdt_status_t destroy_layout(hdt_layout_t *layout, bool completed)
{
    if (!layout) return HDT_OK;
    if (layout->magic != HDT_LAYOUT_MAGIC) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_layout_destroy: not a layout");
    // the build and every attention call went through this handle: its streams cover the layouts it owns
    const HdtUsers users = completed ? HdtUsers() : hdt_users_at_release(hdt_layout_streams(layout));
    hdt_layout_t *owned[3] = {layout->compact ? layout->compact->transposed : nullptr, layout->compact, layout->transposed};
    layout->compact = layout->transposed = nullptr;
    for (hdt_layout_t *t : owned) {
        if (!t) continue;
        t->transposed = nullptr;
        t->magic = 0;
        hdt_layout_release(t, users);
        delete t;
    }
    layout->magic = 0;
    hdt_layout_release(layout, users);
    delete layout;
    return HDT_OK;
}

extern "C" __attribute__((visibility("default"))) hdt_status_t hdt_layout_destroy(hdt_layout_t *layout)
{
    return destroy_layout(layout, false);
}

extern "C" __attribute__((visibility("default"))) hdt_status_t hdt_layout_destroy_completed(hdt_layout_t *layout)
{
    return destroy_layout(layout, true);
}

// ---------------------------------------------------------------------------- attention
static hdt_status_t check_attn_args(const char *fn, const hdt_layout_t *layout, int32_t heads, int32_t head_dim,
                                    hdt_dtype_t dt, float scale)
{
    if (!hdt_layout_ok(layout)) return hdt_fail(HDT_ERR_INVALID_ARG, "%s: NULL or invalid layout", fn);
    if (heads < 0) return hdt_fail(HDT_ERR_INVALID_ARG, "%s: heads = %d", fn, heads);
    if (!(scale > 0.f) || !isfinite(scale))
        return hdt_fail(HDT_ERR_INVALID_ARG, "%s: softmax_scale must be positive and finite", fn);
    if (dt != HDT_BF16 && dt != HDT_F32) return hdt_fail(HDT_ERR_UNSUPPORTED, "%s: unknown dtype %d", fn, (int)dt);
    if (head_dim != 64 && head_dim != 128)
        return hdt_fail(HDT_ERR_UNSUPPORTED, "%s: head_dim %d (supported: 64, 128)", fn, head_dim);
    if (dt == HDT_BF16 && !((layout->s.bm == 64 && layout->s.bn == 32) || (layout->s.bm == 128 && layout->s.bn == 64)))
        return hdt_fail(HDT_ERR_UNSUPPORTED, "%s: bf16 kernels need 64x32 or 128x64 tiles, layout has %dx%d", fn,
                        layout->s.bm, layout->s.bn);
    // a deferred build that is known to have failed (a look at its report, no wait)
    return hdt_layout_resolve(layout, false);
}

static bool misaligned(const void *p) { return ((uintptr_t)p & 15u) != 0; }

extern "C" __attribute__((visibility("default"))) size_t hdt_attn_fwd_workspace_bytes(const hdt_layout_t *layout, int32_t heads,
                                                                                       int32_t head_dim, hdt_dtype_t dt)
{
    if (!hdt_layout_ok(layout) || heads <= 0 || dt != HDT_BF16 || (head_dim != 64 && head_dim != 128)) return 0;
    return hdt_cross_fwd_workspace_bytes(layout, heads, head_dim);
}

extern "C" __attribute__((visibility("default"))) hdt_status_t hdt_attn_fwd(const hdt_layout_t *layout, const void *q, const void *k, const void *v,
                                     void *o, float *lse, int32_t heads, int32_t head_dim, hdt_dtype_t dt,
                                     float scale, void *stream)
{
    return hdt_attn_fwd_ws(layout, q, k, v, o, lse, heads, head_dim, dt, scale, nullptr, 0, stream);
}

extern "C" __attribute__((visibility("default"))) hdt_status_t hdt_attn_fwd_ws(const hdt_layout_t *layout, const void *q, const void *k,
                                                                                const void *v, void *o, float *lse, int32_t heads,
                                                                                int32_t head_dim, hdt_dtype_t dt, float scale,
                                                                                void *workspace, size_t workspace_bytes, void *stream)
{
    hdt_status_t st = check_attn_args("hdt_attn_fwd", layout, heads, head_dim, dt, scale);
    if (st != HDT_OK) return st;
    const HdtSchedule &s = layout->s;
    if (s.batch == 0 || s.n_pos == 0 || heads == 0) return HDT_OK;
    if (!q || !k || !v || !o || !lse) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_attn_fwd: NULL tensor pointer");
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o) || ((uintptr_t)lse & 3u))
        return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_attn_fwd: tensor pointers must be 16-byte aligned");
    if (o == q || o == k || o == v) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_attn_fwd: output aliases an input");
    if ((int64_t)s.batch * heads * s.tr > 0x7ffff000LL)
        return hdt_fail(HDT_ERR_SHAPE, "hdt_attn_fwd: batch*heads*q_tiles exceeds the grid limit");
    hipStream_t hs = (hipStream_t)stream;
    hdt_layout_note_stream(layout, hs);  // whoever gets this layout's buffers later waits for this stream
    // long key lists of a cross-attention layout, cut into pieces, when the caller brings room for the partial results
    const size_t ws_need = dt == HDT_BF16 ? hdt_cross_fwd_workspace_bytes(layout, heads, head_dim) : 0;
    if (ws_need > 0 && workspace != nullptr && workspace_bytes >= ws_need) {
        if (misaligned(workspace)) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_attn_fwd_ws: the workspace must be 16-byte aligned");
        return hdt_cross_fwd_split(layout, q, k, v, o, lse, heads, head_dim, scale, workspace, hs);
    }
    if (dt == HDT_BF16) return hdt_launch_fwd_bf16(s, q, k, v, o, lse, heads, head_dim, scale, hs);
    return hdt_launch_fwd_f32(s, (const float *)q, (const float *)k, (const float *)v, (float *)o, lse, heads,
                              head_dim, scale, hs);
}

extern "C" __attribute__((visibility("default"))) size_t hdt_attn_bwd_workspace_bytes(const hdt_layout_t *layout, int32_t heads, int32_t head_dim,
                                               hdt_dtype_t dt)
{
    if (!hdt_layout_ok(layout) || heads < 0) return 0;
    // two floats per (batch, head, position): D_i = sum_c dO_ic O_ic and LSE_i in the form the kernels start from
    size_t n = hdt_bwd_row_scalars_bytes((size_t)layout->s.batch * (size_t)heads * (size_t)layout->s.n_pos);
    // a cross-attention layout with a compact pair: compact copies of K, V and of their gradients behind it
    if (layout->compact) n += hdt_cross_compact_workspace_bytes(layout, heads, head_dim, dt == HDT_BF16 ? 2 : 4);
    // a cross-attention layout with long key lists: the parts of dQ that the pieces of the lists produce
    if (dt == HDT_BF16 && (head_dim == 64 || head_dim == 128)) n += hdt_cross_dq_workspace_bytes(layout, heads, head_dim);
    return n;
}

// ---- hdt_attn_bwd for callers that cannot allocate: the workspace is an array of the library's own ----
// One copy per GPU, alive until the process ends.  In host code the array's name only stands for the symbol;
// its address on the current device comes from hipGetSymbolAddress, once per device.
static __device__ __align__(256) unsigned char scratch[HDT_NO_ALLOC_WORKSPACE_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

hdt_status_t scratch_on_current_device(void **out)
{
    int dev = 0;
    HDT_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return hdt_fail(HDT_ERR_UNSUPPORTED, "hdt_attn_bwd_no_alloc: device %d", dev);
    std::lock_guard<std::mutex> lk(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        HDT_HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return hdt_fail(HDT_ERR_HIP, "hdt_attn_bwd_no_alloc: the scratch array has no address on device %d", dev);
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return HDT_OK;
}
}  // namespace

extern "C" __attribute__((visibility("default"))) hdt_status_t hdt_attn_bwd_no_alloc(
    const hdt_layout_t *layout, const void *q, const void *k, const void *v, const void *o, const float *lse,
    const void *d_o, void *dq, void *dk, void *dv, int32_t heads, int32_t head_dim, hdt_dtype_t dt, float scale,
    void *stream)
{
    hdt_status_t st = check_attn_args("hdt_attn_bwd_no_alloc", layout, heads, head_dim, dt, scale);
    if (st != HDT_OK) return st;
    if (layout->s.batch == 0 || layout->s.n_pos == 0 || heads == 0) return HDT_OK;
    const size_t need = hdt_attn_bwd_workspace_bytes(layout, heads, head_dim, dt);
    if (need > (size_t)HDT_NO_ALLOC_WORKSPACE_BYTES)
        return hdt_fail(HDT_ERR_SHAPE,
                        "hdt_attn_bwd_no_alloc: this call needs %zu bytes of workspace, the library's own array holds %zu "
                        "(batch * heads * n_pos <= %zu for a self-attention layout); use hdt_attn_bwd",
                        need, (size_t)HDT_NO_ALLOC_WORKSPACE_BYTES, (size_t)HDT_NO_ALLOC_WORKSPACE_BYTES / sizeof(float));
    void *ws = nullptr;
    st = scratch_on_current_device(&ws);
    if (st != HDT_OK) return st;
    return hdt_attn_bwd(layout, q, k, v, o, lse, d_o, dq, dk, dv, heads, head_dim, dt, scale, ws,
                        (size_t)HDT_NO_ALLOC_WORKSPACE_BYTES, stream);
}

extern "C" __attribute__((visibility("default"))) hdt_status_t hdt_attn_bwd(const hdt_layout_t *layout, const void *q, const void *k, const void *v,
                                     const void *o, const float *lse, const void *d_o, void *dq, void *dk,
                                     void *dv, int32_t heads, int32_t head_dim, hdt_dtype_t dt, float scale,
                                     void *workspace, size_t workspace_bytes, void *stream)
{
    hdt_status_t st = check_attn_args("hdt_attn_bwd", layout, heads, head_dim, dt, scale);
    if (st != HDT_OK) return st;
    const HdtSchedule &s = layout->s;
    const HdtSchedule &s_tr = layout->transposed ? layout->transposed->s : s;
    if (s.batch == 0 || s.n_pos == 0 || heads == 0) return HDT_OK;
    if (!q || !k || !v || !o || !lse || !d_o || !dq || !dk || !dv)
        return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_attn_bwd: NULL tensor pointer");
    const void *ptrs[] = {q, k, v, o, d_o, dq, dk, dv, workspace};
    for (const void *p : ptrs)
        if (misaligned(p)) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_attn_bwd: pointers must be 16-byte aligned");
    const void *ins[] = {q, k, v, o, d_o};
    void *outs[] = {dq, dk, dv};
    for (void *w : outs) {
        for (const void *r : ins)
            if (w == r) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_attn_bwd: output aliases an input");
    }
    if (dq == dk || dq == dv || dk == dv) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_attn_bwd: outputs alias each other");
    size_t need = hdt_attn_bwd_workspace_bytes(layout, heads, head_dim, dt);
    if (!workspace || workspace_bytes < need)
        return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_attn_bwd: workspace of %zu bytes needed, %zu given", need,
                        workspace_bytes);
    if ((int64_t)s.batch * heads * ((int64_t)s.tr + 2 * (int64_t)s_tr.tr) > 0x7ffff000LL)
        return hdt_fail(HDT_ERR_SHAPE, "hdt_attn_bwd: batch*heads*tiles exceeds the grid limit");
    hipStream_t hs = (hipStream_t)stream;
    hdt_layout_note_stream(layout, hs);
    if (layout->compact)
        return hdt_cross_bwd_compact(layout, q, k, v, o, lse, d_o, dq, dk, dv, heads, head_dim, dt == HDT_BF16, scale,
                                     workspace, hs);
    if (dt == HDT_BF16 && hdt_cross_pieces(layout, heads) > 1)
        return hdt_cross_bwd_split(layout, q, k, v, o, lse, d_o, dq, dk, dv, heads, head_dim, scale, workspace, hs);
    if (dt == HDT_BF16)
        return hdt_launch_bwd_bf16(s, s_tr, q, k, v, o, lse, d_o, dq, dk, dv, heads, head_dim, scale, (float *)workspace, hs);
    return hdt_launch_bwd_f32(s, s_tr, (const float *)q, (const float *)k, (const float *)v, (const float *)o, lse,
                              (const float *)d_o, (float *)dq, (float *)dk, (float *)dv, heads, head_dim, scale,
                              (float *)workspace, hs);
}
