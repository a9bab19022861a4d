// hdt_build_cross_layout: the schedule of decoder cross-attention over a level subset of the encoder's
// positions (Sec. 4.2, FacetSum study: the decoder attends only to the [SEC] anchors, or additionally to
// the [SENT] anchors, or additionally to the regular tokens).
//
// The mask is a rectangle: every decoder row may attend to every visible encoder position (non-pad, level
// in the given set).  In the terms of the attention kernels that is a key list per row tile, the same for
// all row tiles of a sample: the visible positions in document order, tile_n per list entry.  So the
// "gather of the anchor rows" is the gather the attention kernels do anyway, straight into LDS; no compacted
// copy of K and V is made.  The backward pass needs the transposed schedule as well: rows are the encoder
// positions (allowed iff visible), a row tile that holds a visible position lists all decoder rows.
//
// The list entries of a row tile sit at a fixed stride (room for the longest possible list), the unused ones
// are marked empty, and a tile's range covers the ones in use.
//
// The dK/dV pass of the backward tiles the ENCODER rows, and with a few anchors visible nearly every 32-row
// block of them holds one allowed row among 31 idle ones.  The build therefore reads the number of visible
// positions back, and when they are at most a quarter of the encoder's positions it adds a second pair of
// schedules in the index space of the visible positions (row = rank among them): hdt_attn_bwd then gathers
// the visible rows of K and V into compact tensors (in its workspace), runs the ordinary backward kernels
// on those, and scatters dK and dV back (zeros for the rows that are not visible).  The forward keeps
// gathering straight from K and V.
//
// With the regular tokens visible the opposite happens: a handful of decoder row tiles each walk a key list of
// more than a hundred entries one after the other, on a few workgroups.  The list of a row tile is the same for
// every row tile of a sample, so cutting it costs nothing but a second table of entry ranges: with the lists cut
// into P pieces the forward (and the dQ role of the backward) see P times the row tiles, piece p of tile I
// covering entries [p * chunk, (p + 1) * chunk) of the tile's list and producing a partial result for the tile's
// rows (O and LSE over its keys; its part of dQ), and a small kernel puts the pieces together in a fixed order
// (O = sum_p w_p O_p with w_p = exp(LSE_p - LSE), LSE = log sum_p exp(LSE_p); dQ = sum_p dQ_p).  The partial
// results live in the caller's workspace (hdt_attn_fwd_ws, hdt_attn_bwd).
#include <string.h>

#include <initializer_list>
#include <new>
#include <vector>

#include "hdt_internal.h"

namespace {

constexpr int kSelThreads = 1024;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ bool visible(int level, uint32_t level_mask)
{
    return level >= 0 && level < 32 && ((level_mask >> level) & 1u);
}

// One workgroup per sample: the visible positions in document order (sel) and their number (count).
__global__ __launch_bounds__(kSelThreads) void k_cross_select(const int32_t *__restrict__ level, int n_enc,
                                                               uint32_t level_mask, int32_t *__restrict__ sel,
                                                               int32_t *__restrict__ rank, int32_t *__restrict__ count)
{
    __shared__ int s_wave[kSelThreads / 64];
    __shared__ int s_base;
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int32_t *lv = level + (size_t)b * n_enc;
    int32_t *out = sel + (size_t)b * n_enc;
    if (tid == 0) s_base = 0;
    __syncthreads();
    for (int i0 = 0; i0 < n_enc; i0 += kSelThreads) {
        const int i = i0 + tid;
        const bool vis = i < n_enc && visible(lv[i], level_mask);
        const unsigned long long m = __ballot(vis);
        if (lane == 0) s_wave[wave] = __popcll(m);
        __syncthreads();
        int before = s_base;
        for (int w = 0; w < wave; w++) before += s_wave[w];
        const int mine = before + __popcll(m & ((1ull << lane) - 1ull));
        if (vis) out[mine] = i;
        if (i < n_enc) rank[(size_t)b * n_enc + i] = vis ? mine : -1;
        __syncthreads();
        if (tid == 0) {
            int tot = 0;
            for (int w = 0; w < kSelThreads / 64; w++) tot += s_wave[w];
            s_base += tot;
        }
        __syncthreads();
    }
    if (tid == 0) count[b] = s_base;
}

struct CrossArgs {
    const int32_t *level;  // [B][n_enc]
    const int32_t *sel;    // [B][n_enc] visible positions
    const int32_t *count;  // [B]
    uint32_t level_mask;
    int n_enc, n_dec, bm, bn;
    int transposed;  // 0: rows = decoder positions, keys = visible encoder positions; 1: rows = encoder positions
                     // (allowed iff visible), keys = decoder positions
    int tr, e_max;   // row tiles per sample, list entries reserved per row tile
    int compact;     // 0, or the rows per sample of the compact tensors: encoder positions are named by their rank
                     // among the visible ones (keys of the forward schedule, rows of the transposed one)
    int32_t *q_range, *c_row, *c_cnt, *q_keys;
    uint32_t *q_sub;
    unsigned long long *bits_rm;
};

// One wave per reserved list entry (b, I, e): its keys, bitmaps and summary, or the "empty" marks.
__global__ __launch_bounds__(64) void k_cross_entries(CrossArgs a)
{
    __shared__ uint32_t s_row[4], s_col[4];  // allowed rows / filled key slots of the entry, bit masks
    const int lane = threadIdx.x;
    const int e = blockIdx.x % a.e_max, tile = blockIdx.x / a.e_max;  // tile = b * tr + I
    const int b = tile / a.tr, I = tile % a.tr;
    const int64_t entry = blockIdx.x;
    const int n_rows = a.transposed ? (a.compact ? a.compact : a.n_enc) : a.n_dec;
    const int n_keys = a.transposed ? a.n_dec : a.count[b];
    // rows of the tile
    bool any_row = false;
    for (int h = 0; h < 2; h++) {
        const int r = h * 64 + lane, i = I * a.bm + r;
        bool ok = r < a.bm && i < n_rows;
        if (ok && a.transposed) ok = a.compact ? i < a.count[b] : visible(a.level[(size_t)b * a.n_enc + i], a.level_mask);
        const unsigned long long m = __ballot(ok);
        if (lane == 0) {
            s_row[2 * h] = (uint32_t)m;
            s_row[2 * h + 1] = (uint32_t)(m >> 32);
        }
        any_row |= m != 0ull;
    }
    const int n_ent = (a.transposed && !any_row) ? 0 : (n_keys + a.bn - 1) / a.bn;
    if (e == 0 && lane == 0) {
        a.q_range[2 * tile] = (int32_t)entry;
        a.q_range[2 * tile + 1] = (int32_t)entry + n_ent;
    }
    if (lane == 0) a.c_row[entry] = tile;
    if (e >= n_ent) {  // reserved, not in use
        if (lane == 0) {
            a.c_cnt[entry] = 0;
            a.q_sub[entry] = 0u;
        }
        return;
    }
    // key slots
    for (int h = 0; h < 2; h++) {
        const int c = h * 64 + lane, idx = e * a.bn + c;
        const bool ok = c < a.bn && idx < n_keys;
        // a slot past the last key holds ~f, f = the entry's first key: the row gathered in its place
        const int at = ok ? idx : e * a.bn;
        const int key = (a.transposed || a.compact) ? at : a.sel[(size_t)b * a.n_enc + at];
        if (c < a.bn) a.q_keys[entry * a.bn + c] = ok ? key : ~key;
        const unsigned long long m = __ballot(ok);
        if (lane == 0) {
            s_col[2 * h] = (uint32_t)m;
            s_col[2 * h + 1] = (uint32_t)(m >> 32);
        }
    }
    __syncthreads();
    const int wpr = a.bn >> 5, nrb = a.bm >> 5, nsub = nrb * wpr;
    // lane masks of the MFMA accumulator registers: sub-block (rblk, cblk), register x: bit l <=> row
    // rblk*32 + l%32, column cblk*32 + (l/32)*4 + 8*(x/4) + x%4
    for (int w = lane; w < nsub * 16; w += 64) {
        const int sb = w >> 4, x = w & 15, rblk = sb / wpr, cblk = sb % wpr;
        const uint32_t rows = s_row[rblk], cols = s_col[cblk];
        unsigned long long m = 0;
        for (int h = 0; h < 2; h++) {
            const int col = h * 4 + 8 * (x >> 2) + (x & 3);
            if ((cols >> col) & 1u) m |= (unsigned long long)rows << (32 * h);
        }
        a.bits_rm[((size_t)entry * nsub + sb) * 16 + x] = m;
    }
    if (lane == 0) {
        uint32_t any = 0, all = 0;
        int nr = 0, nc = 0;
        for (int i = 0; i < 4; i++) {
            nr += __popc(s_row[i]);
            nc += __popc(s_col[i]);
        }
        for (int rblk = 0; rblk < nrb; rblk++)
            for (int cblk = 0; cblk < wpr; cblk++) {
                const int sb = rblk * wpr + cblk;
                if (s_row[rblk] != 0u && s_col[cblk] != 0u) any |= 1u << sb;
                if (s_row[rblk] == 0xffffffffu && s_col[cblk] == 0xffffffffu) all |= 1u << sb;
            }
        a.c_cnt[entry] = nr * nc;
        a.q_sub[entry] = any | (all << 16);
    }
}

// ---- compact copies for the backward: rows of [B][H][n][row_bytes] tensors, 16 bytes per thread ----------
// dst[b][h][c] = src[b][h][sel[b][c]] for c < count[b], zeros for the other rows of the compact tensors
// (they are operands of the kernels' contractions, masked but read); two tensors per launch.
__global__ __launch_bounds__(256) void k_cross_gather(const int32_t *__restrict__ sel, const int32_t *__restrict__ count,
                                                       int n_enc, int n_compact, int heads, int chunks,
                                                       const u32x4 *__restrict__ src0, const u32x4 *__restrict__ src1,
                                                       u32x4 *__restrict__ dst0, u32x4 *__restrict__ dst1, long long total)
{
    const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
    if (t >= total) return;
    const int ch = (int)(t % chunks);
    const long long row = t / chunks;  // (b * heads + h) * n_compact + c
    const int c = (int)(row % n_compact);
    const long long bh = row / n_compact;
    const int b = (int)(bh / heads);
    u32x4 x0 = {0u, 0u, 0u, 0u}, x1 = x0;
    if (c < count[b]) {
        const long long from = (bh * n_enc + sel[(size_t)b * n_enc + c]) * chunks + ch;
        x0 = src0[from];
        x1 = src1[from];
    }
    dst0[t] = x0;
    dst1[t] = x1;
}

// dst[b][h][p] = src[b][h][rank[b][p]] for visible p, zeros otherwise; two tensors per launch
__global__ __launch_bounds__(256) void k_cross_scatter(const int32_t *__restrict__ rank, int n_enc, int n_compact, int heads,
                                                        int chunks, const u32x4 *__restrict__ src0,
                                                        const u32x4 *__restrict__ src1, u32x4 *__restrict__ dst0,
                                                        u32x4 *__restrict__ dst1, long long total)
{
    const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
    if (t >= total) return;
    const int ch = (int)(t % chunks);
    const long long row = t / chunks;  // (b * heads + h) * n_enc + p
    const int pos = (int)(row % n_enc);
    const long long bh = row / n_enc;
    const int b = (int)(bh / heads);
    const int r = rank[(size_t)b * n_enc + pos];
    u32x4 x0 = {0u, 0u, 0u, 0u}, x1 = x0;
    if (r >= 0) {
        const long long from = (bh * n_compact + r) * chunks + ch;
        x0 = src0[from];
        x1 = src1[from];
    }
    __builtin_nontemporal_store(x0, &dst0[t]);
    __builtin_nontemporal_store(x1, &dst1[t]);
}

// Entry ranges of the forward schedule with every key list cut into `pieces`: row tile p * tr + I of sample b gets
// entries [p * chunk, (p + 1) * chunk) of the list of tile (b, I), chunk = ceil(entries / pieces).
__global__ __launch_bounds__(256) void k_cross_split_ranges(const int32_t *__restrict__ count, int batch, int tr, int bn,
                                                             int e_max, int pieces, int32_t *__restrict__ out)
{
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= batch * pieces * tr) return;
    const int b = t / (pieces * tr), r = t % (pieces * tr), p = r / tr, I = r % tr;
    const int n_ent = (count[b] + bn - 1) / bn, chunk = (n_ent + pieces - 1) / pieces;
    const int first = min(p * chunk, n_ent), last = min(first + chunk, n_ent);
    const int base = (b * tr + I) * e_max;
    out[2 * t] = base + first;
    out[2 * t + 1] = base + last;
}

// O, LSE of row (bh, r) from the partial results of the pieces: o_part [bh][PIECES * rows_pad][D] bf16 (piece p of
// row r at p * rows_pad + r), lse_part [bh][PIECES * rows_pad].  One thread per 8 columns; all loads of a thread are
// issued before the first is used.
template <int D, int PIECES>
__global__ __launch_bounds__(256) void k_cross_combine_fwd(const u32x4 *__restrict__ o_part, const float *__restrict__ lse_part,
                                                            u32x4 *__restrict__ o, float *__restrict__ lse, int n_rows,
                                                            int rows_pad, long long total)
{
    constexpr int CPR = D / 8;
    const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
    if (t >= total) return;
    const int c = (int)(t % CPR);
    const long long row = t / CPR;  // bh * n_rows + r
    const int r = (int)(row % n_rows);
    const long long bh = row / n_rows;
    const size_t prow = (size_t)bh * PIECES * rows_pad + r;
    float l[PIECES];
    u32x4 x[PIECES];
#pragma unroll
    for (int p = 0; p < PIECES; p++) {
        l[p] = lse_part[prow + (size_t)p * rows_pad];
        x[p] = o_part[(prow + (size_t)p * rows_pad) * CPR + c];
    }
    float m = -INFINITY;
#pragma unroll
    for (int p = 0; p < PIECES; p++) m = fmaxf(m, l[p]);
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, z = 0.f;
#pragma unroll
    for (int p = 0; p < PIECES; p++) {
        // a piece without keys has LSE = -inf and rows of zeros: weight 0
        const float w = (m == -INFINITY || l[p] == -INFINITY) ? 0.f : __expf(l[p] - m);
        z += w;
#pragma unroll
        for (int e = 0; e < 4; e++) {
            acc[2 * e] += w * __uint_as_float(x[p][e] << 16);
            acc[2 * e + 1] += w * __uint_as_float(x[p][e] & 0xffff0000u);
        }
    }
    const float inv = z > 0.f ? 1.f / z : 0.f;
    u32x4 y;
#pragma unroll
    for (int e = 0; e < 4; e++) {
        const __bf16 lo = (__bf16)(acc[2 * e] * inv), hi = (__bf16)(acc[2 * e + 1] * inv);
        y[e] = (uint32_t)__builtin_bit_cast(unsigned short, lo) | ((uint32_t)__builtin_bit_cast(unsigned short, hi) << 16);
    }
    o[row * CPR + c] = y;
    if (c == 0) lse[row] = z > 0.f ? m + __logf(z) : -INFINITY;
}

// dQ of row (bh, r) = the sum of the pieces' parts, in piece order
template <int D, int PIECES>
__global__ __launch_bounds__(256) void k_cross_sum_dq(const u32x4 *__restrict__ dq_part, u32x4 *__restrict__ dq, int n_rows,
                                                       int rows_pad, long long total)
{
    constexpr int CPR = D / 8;
    const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
    if (t >= total) return;
    const int c = (int)(t % CPR);
    const long long row = t / CPR;
    const int r = (int)(row % n_rows);
    const long long bh = row / n_rows;
    const size_t prow = (size_t)bh * PIECES * rows_pad + r;
    u32x4 x[PIECES];
#pragma unroll
    for (int p = 0; p < PIECES; p++) x[p] = dq_part[(prow + (size_t)p * rows_pad) * CPR + c];
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int p = 0; p < PIECES; p++) {
#pragma unroll
        for (int e = 0; e < 4; e++) {
            acc[2 * e] += __uint_as_float(x[p][e] << 16);
            acc[2 * e + 1] += __uint_as_float(x[p][e] & 0xffff0000u);
        }
    }
    u32x4 y;
#pragma unroll
    for (int e = 0; e < 4; e++) {
        const __bf16 lo = (__bf16)acc[2 * e], hi = (__bf16)acc[2 * e + 1];
        y[e] = (uint32_t)__builtin_bit_cast(unsigned short, lo) | ((uint32_t)__builtin_bit_cast(unsigned short, hi) << 16);
    }
    dq[row * CPR + c] = y;
}

struct CrossBuffers {
    int32_t *split_range[3];                // first arena, forward schedule only: entry ranges with the lists cut in 2, 4, 8
    int32_t *sel, *rank, *count, *q_range;  // first arena
    int32_t *c_row, *c_cnt, *q_keys;  // second arena
    uint32_t *q_sub;
    unsigned long long *bits_rm;
    size_t bytes1, bytes2;
};

template <typename T>
T *carve(char *base, size_t &off, size_t count)
{
    T *p = base ? reinterpret_cast<T *>(base + off) : nullptr;
    off += (count * sizeof(T) + 255) & ~(size_t)255;
    return p;
}

CrossBuffers carve_cross(char *a1, char *a2, int B, int n_enc, int tr, int64_t entries, int bm, int bn, bool with_sel)
{
    CrossBuffers c{};
    size_t o1 = 0, o2 = 0;
    if (with_sel) {
        c.sel = carve<int32_t>(a1, o1, (size_t)B * n_enc);
        c.rank = carve<int32_t>(a1, o1, (size_t)B * n_enc);
        c.count = carve<int32_t>(a1, o1, (size_t)B);
        for (int k = 0; k < 3; k++) c.split_range[k] = carve<int32_t>(a1, o1, (size_t)B * tr * (2 << k) * 2);
    }
    c.q_range = carve<int32_t>(a1, o1, (size_t)B * tr * 2);
    const size_t n = (size_t)entries;
    c.c_row = carve<int32_t>(a2, o2, n);
    c.c_cnt = carve<int32_t>(a2, o2, n);
    c.q_sub = carve<uint32_t>(a2, o2, n);
    c.q_keys = carve<int32_t>(a2, o2, n * (size_t)bn);
    c.bits_rm = carve<unsigned long long>(a2, o2, n * (size_t)(bm / 32) * (bn / 32) * 16);
    c.bytes1 = o1;
    c.bytes2 = o2;
    return c;
}

hdt_layout_t *new_layout(int batch, int n_rows, int n_kv, int bm, int bn)
{
    hdt_layout_t *L = new (std::nothrow) hdt_layout_t();
    if (!L) return nullptr;
    L->magic = HDT_LAYOUT_MAGIC;
    L->arena = L->arena2 = nullptr;
    L->arena_bytes = L->arena2_bytes = 0;
    L->capacity = 0;
    L->d_cnt = L->d_row = nullptr;
    L->n_entries = 0;
    L->stats_ready = false;
    L->kperm_ready = true;
    L->no_sort = 0;
    L->sort_hist = L->sort_counters = nullptr;
    L->level_copy = L->parent_copy = nullptr;
    L->force_dense = 0;
    L->windowed = 0;
    L->edges = 0;
    L->cross = 1;
    L->transposed = nullptr;
    L->compact = nullptr;
    L->cross_sel = L->cross_count = L->cross_rank = nullptr;
    L->n_compact = 0;
    for (auto &r : L->cross_split_range) r = nullptr;
    L->cross_entries_max = 0;
    L->device_bytes = 0;
    L->device = 0;
    (void)hipGetDevice(&L->device);
    HdtSchedule &s = L->s;
    memset(&s, 0, sizeof(s));
    s.batch = batch;
    s.n_pos = n_rows;
    s.n_kv = n_kv;
    s.bm = bm;
    s.bn = bn;
    s.wpr = bn / 32;
    s.tr = (n_rows + bm - 1) / bm;
    s.tc = (n_kv + bn - 1) / bn;
    s.n_slots = s.tc * bn;
    s.n_own = n_rows;
    s.tr_own = s.tr;
    L->h_stats.assign((size_t)batch * 2, 0);
    return L;
}

// the finished arrays become the layout's schedule
void adopt(hdt_layout_t *l, const CrossBuffers &c, int64_t n)
{
    HdtSchedule &s = l->s;
    s.q_range = c.q_range;
    s.q_keys = c.q_keys;
    s.q_sub = c.q_sub;
    s.bits_rm = c.bits_rm;
    s.q_cols = nullptr;
    s.kperm = nullptr;
    l->d_cnt = c.c_cnt;
    l->d_row = c.c_row;
    l->n_entries = n;
    l->capacity = n;
    l->device_bytes = (int64_t)(l->arena_bytes + l->arena2_bytes);
    if (n == 0) l->stats_ready = true;
}

}  // namespace

extern "C" __attribute__((visibility("default"))) hdt_status_t hdt_build_cross_layout(
    const int32_t *d_level_enc, int32_t batch, int32_t n_enc, int32_t n_dec, uint32_t level_mask,
    const hdt_layout_opts_t *opts, void *stream, hdt_layout_t **out)
{
    if (!out) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_build_cross_layout: out is NULL");
    *out = nullptr;
    if (batch < 0 || n_enc < 0 || n_dec < 0) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_build_cross_layout: negative size");
    if (n_enc > (1 << 19) || n_dec > (1 << 19))
        return hdt_fail(HDT_ERR_SHAPE, "hdt_build_cross_layout: n_enc %d or n_dec %d > 2^19", n_enc, n_dec);
    int bm = 128, bn = 64;
    if (opts) {
        if (opts->tile_m) bm = opts->tile_m;
        if (opts->tile_n) bn = opts->tile_n;
        if (opts->force_dense || opts->no_sort || opts->windowed || opts->edges || opts->deferred || opts->capacity)
            return hdt_fail(HDT_ERR_UNSUPPORTED, "hdt_build_cross_layout: only the tile shape can be chosen");
    }
    if (bm < 32 || bm > 128 || bm % 32 || bn < 32 || bn > 128 || bn % 32)
        return hdt_fail(HDT_ERR_UNSUPPORTED, "hdt_build_cross_layout: tile %dx%d (each side: 32, 64, 96 or 128)", bm, bn);
    if (batch > 0 && (n_enc == 0 || n_dec == 0))
        return hdt_fail(HDT_ERR_SHAPE, "hdt_build_cross_layout: n_enc = %d, n_dec = %d (both sides need rows)", n_enc, n_dec);
    const bool empty = batch == 0;
    if (!empty && !d_level_enc) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_build_cross_layout: NULL level array");

    hdt_layout_t *L = new_layout(batch, n_dec, n_enc, bm, bn);
    hdt_layout_t *T = L ? new_layout(batch, n_enc, n_dec, bm, bn) : nullptr;
    if (!L || !T) {
        delete L;
        return hdt_fail(HDT_ERR_OOM, "hdt_build_cross_layout: host allocation failed");
    }
    L->transposed = T;
    L->cross_level_mask = T->cross_level_mask = level_mask;
    hdt_layout_t *Lc = nullptr, *Tc = nullptr;  // the compact pair while it is being built
    hdt_status_t status = HDT_OK;
    hipStream_t st = (hipStream_t)stream;
    L->streams.add(st);
    hdt_note_build_stream(st);
    HdtUsers build_only;  // what the buffers of a failed build have been touched by
    build_only.lazy.add(st);
    const int e_fwd = (n_enc + bn - 1) / bn, e_tr = (n_dec + bn - 1) / bn;
    const int64_t ent_fwd = (int64_t)batch * L->s.tr * e_fwd, ent_tr = (int64_t)batch * T->s.tr * e_tr;
    if (ent_fwd >= (1LL << 31) || ent_tr >= (1LL << 31)) {
        status = hdt_fail(HDT_ERR_SHAPE, "hdt_build_cross_layout: %lld list entries", (long long)(ent_fwd > ent_tr ? ent_fwd : ent_tr));
        goto fail;
    }
#define CROSS_TRY(expr)                                                                                \
    do {                                                                                               \
        hipError_t _e = (expr);                                                                        \
        if (_e != hipSuccess) {                                                                        \
            status = hdt_fail(_e == hipErrorOutOfMemory ? HDT_ERR_OOM : HDT_ERR_HIP, "%s: %s", #expr, \
                              hipGetErrorString(_e));                                                  \
            goto fail;                                                                                 \
        }                                                                                              \
    } while (0)
    {
        CrossBuffers f = carve_cross(nullptr, nullptr, batch, n_enc, L->s.tr, ent_fwd, bm, bn, true);
        CrossBuffers t = carve_cross(nullptr, nullptr, batch, n_enc, T->s.tr, ent_tr, bm, bn, false);
        CROSS_TRY(hdt_pool_alloc(&L->arena, f.bytes1 + 256, &L->arena_bytes, st));
        CROSS_TRY(hdt_pool_alloc(&L->arena2, f.bytes2 + 256, &L->arena2_bytes, st));
        CROSS_TRY(hdt_pool_alloc(&T->arena, t.bytes1 + 256, &T->arena_bytes, st));
        CROSS_TRY(hdt_pool_alloc(&T->arena2, t.bytes2 + 256, &T->arena2_bytes, st));
        f = carve_cross((char *)L->arena, (char *)L->arena2, batch, n_enc, L->s.tr, ent_fwd, bm, bn, true);
        t = carve_cross((char *)T->arena, (char *)T->arena2, batch, n_enc, T->s.tr, ent_tr, bm, bn, false);
        if (!empty) {
            {
                HdtTimer tm("hdt_cross_select", st);
                hipLaunchKernelGGL(k_cross_select, dim3((unsigned)batch), dim3(kSelThreads), 0, st, d_level_enc, n_enc,
                                   level_mask, f.sel, f.rank, f.count);
            }
            CrossArgs a{d_level_enc, f.sel, f.count, level_mask, n_enc, n_dec, bm, bn, 0, L->s.tr, e_fwd, 0,
                        f.q_range, f.c_row, f.c_cnt, f.q_keys, f.q_sub, f.bits_rm};
            {
                HdtTimer tm("hdt_cross_entries", st);
                hipLaunchKernelGGL(k_cross_entries, dim3((unsigned)ent_fwd), dim3(64), 0, st, a);
            }
            CrossArgs at{d_level_enc, f.sel, f.count, level_mask, n_enc, n_dec, bm, bn, 1, T->s.tr, e_tr, 0,
                         t.q_range, t.c_row, t.c_cnt, t.q_keys, t.q_sub, t.bits_rm};
            {
                HdtTimer tm("hdt_cross_entries_transposed", st);
                hipLaunchKernelGGL(k_cross_entries, dim3((unsigned)ent_tr), dim3(64), 0, st, at);
            }
            CROSS_TRY(hipGetLastError());
            L->cross_sel = f.sel;
            L->cross_rank = f.rank;
            L->cross_count = f.count;
            // How many positions are visible?  (The one read-back of the build: it waits for the select kernel.)
            std::vector<int32_t> h_count((size_t)batch, 0);
            CROSS_TRY(hipMemcpyAsync(h_count.data(), f.count, sizeof(int32_t) * batch, hipMemcpyDeviceToHost, st));
            CROSS_TRY(hipStreamSynchronize(st));
            int c_max = 0;
            for (int32_t c : h_count) c_max = c > c_max ? c : c_max;
            L->cross_entries_max = (c_max + bn - 1) / bn;
            if (L->cross_entries_max >= 16) {  // lists worth cutting: the entry ranges for 2, 4 and 8 pieces
                for (int k = 0; k < 3; k++) {
                    const int pieces = 2 << k, total = batch * pieces * L->s.tr;
                    hipLaunchKernelGGL(k_cross_split_ranges, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, f.count,
                                       batch, L->s.tr, bn, e_fwd, pieces, f.split_range[k]);
                    L->cross_split_range[k] = f.split_range[k];
                }
                CROSS_TRY(hipGetLastError());
            }
            if (c_max > 0 && (int64_t)c_max * 4 <= n_enc) {
                // the compact pair: decoder rows x ranks, and ranks x decoder rows
                const int n_c = (c_max + 31) / 32 * 32;
                Lc = new_layout(batch, n_dec, n_c, bm, bn);
                Tc = Lc ? new_layout(batch, n_c, n_dec, bm, bn) : nullptr;
                if (!Lc || !Tc) {
                    status = hdt_fail(HDT_ERR_OOM, "hdt_build_cross_layout: host allocation failed");
                    goto fail;
                }
                Lc->transposed = Tc;
                Lc->cross_level_mask = Tc->cross_level_mask = level_mask;
                const int e_fc = (n_c + bn - 1) / bn;
                const int64_t ent_fc = (int64_t)batch * Lc->s.tr * e_fc, ent_tc = (int64_t)batch * Tc->s.tr * e_tr;
                CrossBuffers fc = carve_cross(nullptr, nullptr, batch, n_enc, Lc->s.tr, ent_fc, bm, bn, false);
                CrossBuffers tc = carve_cross(nullptr, nullptr, batch, n_enc, Tc->s.tr, ent_tc, bm, bn, false);
                CROSS_TRY(hdt_pool_alloc(&Lc->arena, fc.bytes1 + 256, &Lc->arena_bytes, st));
                CROSS_TRY(hdt_pool_alloc(&Lc->arena2, fc.bytes2 + 256, &Lc->arena2_bytes, st));
                CROSS_TRY(hdt_pool_alloc(&Tc->arena, tc.bytes1 + 256, &Tc->arena_bytes, st));
                CROSS_TRY(hdt_pool_alloc(&Tc->arena2, tc.bytes2 + 256, &Tc->arena2_bytes, st));
                fc = carve_cross((char *)Lc->arena, (char *)Lc->arena2, batch, n_enc, Lc->s.tr, ent_fc, bm, bn, false);
                tc = carve_cross((char *)Tc->arena, (char *)Tc->arena2, batch, n_enc, Tc->s.tr, ent_tc, bm, bn, false);
                CrossArgs ac{d_level_enc, f.sel, f.count, level_mask, n_enc, n_dec, bm, bn, 0, Lc->s.tr, e_fc, n_c,
                             fc.q_range, fc.c_row, fc.c_cnt, fc.q_keys, fc.q_sub, fc.bits_rm};
                {
                    HdtTimer tm("hdt_cross_entries_compact", st);
                    hipLaunchKernelGGL(k_cross_entries, dim3((unsigned)ent_fc), dim3(64), 0, st, ac);
                }
                CrossArgs atc{d_level_enc, f.sel, f.count, level_mask, n_enc, n_dec, bm, bn, 1, Tc->s.tr, e_tr, n_c,
                              tc.q_range, tc.c_row, tc.c_cnt, tc.q_keys, tc.q_sub, tc.bits_rm};
                {
                    HdtTimer tm("hdt_cross_entries_compact_transposed", st);
                    hipLaunchKernelGGL(k_cross_entries, dim3((unsigned)ent_tc), dim3(64), 0, st, atc);
                }
                CROSS_TRY(hipGetLastError());
                adopt(Lc, fc, ent_fc);
                adopt(Tc, tc, ent_tc);
                L->compact = Lc;
                L->n_compact = n_c;
                L->device_bytes += Lc->device_bytes + Tc->device_bytes;
                Lc = Tc = nullptr;  // owned by L from here on
            }
        }
        struct {
            hdt_layout_t *l;
            CrossBuffers *c;
            int64_t n;
        } both[2] = {{L, &f, empty ? 0 : ent_fwd}, {T, &t, empty ? 0 : ent_tr}};
        const int64_t compact_bytes = L->device_bytes;  // added above, if a compact pair was built
        for (auto &x : both) adopt(x.l, *x.c, x.n);
        T->s.row_flag = f.rank;  // encoder rows that are not visible (pads among them) may hold anything
        L->device_bytes += compact_bytes;
        L->device_bytes += T->device_bytes;
        *out = L;
        return HDT_OK;
    }
fail:
    for (hdt_layout_t *x : {Tc, Lc}) {
        if (!x) continue;
        hdt_layout_release(x, build_only);
        x->magic = 0;
        delete x;
    }
    hdt_layout_release(T, build_only);
    T->magic = 0;
    delete T;
    L->transposed = nullptr;
    hdt_layout_release(L, build_only);
    L->magic = 0;
    delete L;
    return status;
#undef CROSS_TRY
}

// ---- backward through the compact pair ------------------------------------------------------------------
static size_t compact_tensor_bytes(const hdt_layout_t *l, int heads, int head_dim, int elem_bytes)
{
    const size_t n = (size_t)l->s.batch * (size_t)heads * (size_t)l->n_compact * (size_t)head_dim * (size_t)elem_bytes;
    return (n + 255) & ~(size_t)255;
}

size_t hdt_cross_compact_workspace_bytes(const hdt_layout_t *l, int heads, int head_dim, int elem_bytes)
{
    return l->compact ? 4 * compact_tensor_bytes(l, heads, head_dim, elem_bytes) : 0;
}

// Workspace: D of the decoder rows (as for every backward), then the compact K, V, dK, dV.  The visible rows of K
// and V are gathered, the ordinary backward runs on the compact pair of schedules (dQ is written in place: its rows
// are the decoder's), and dK, dV are scattered to the encoder's rows, zeros where a row is not visible.
hdt_status_t hdt_cross_bwd_compact(const hdt_layout_t *l, const void *q, const void *k, const void *v, const void *o,
                                   const float *lse, const void *d_o, void *dq, void *dk, void *dv, int heads,
                                   int head_dim, bool bf16, float scale, void *workspace, hipStream_t st)
{
    const hdt_layout_t *lc = l->compact;
    const HdtSchedule &s = lc->s, &s_tr = lc->transposed->s;
    const int elem = bf16 ? 2 : 4, n_enc = l->s.n_kv, n_c = l->n_compact, B = l->s.batch;
    const size_t d_bytes = hdt_bwd_row_scalars_bytes((size_t)B * heads * (size_t)l->s.n_pos);
    const size_t t_bytes = compact_tensor_bytes(l, heads, head_dim, elem);
    char *w = static_cast<char *>(workspace);
    float *delta = reinterpret_cast<float *>(w);
    void *kc = w + d_bytes, *vc = w + d_bytes + t_bytes, *dkc = w + d_bytes + 2 * t_bytes, *dvc = w + d_bytes + 3 * t_bytes;
    const int chunks = head_dim * elem / 16;
    {
        const long long total = (long long)B * heads * n_c * chunks;
        HdtTimer tm("hdt_cross_gather", st);
        hipLaunchKernelGGL(k_cross_gather, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, l->cross_sel, l->cross_count,
                           n_enc, n_c, heads, chunks, (const u32x4 *)k, (const u32x4 *)v, (u32x4 *)kc, (u32x4 *)vc, total);
    }
    HDT_HIP_TRY(hipGetLastError());
    hdt_status_t status =
        bf16 ? hdt_launch_bwd_bf16(s, s_tr, q, kc, vc, o, lse, d_o, dq, dkc, dvc, heads, head_dim, scale, delta, st)
             : hdt_launch_bwd_f32(s, s_tr, (const float *)q, (const float *)kc, (const float *)vc, (const float *)o, lse,
                                  (const float *)d_o, (float *)dq, (float *)dkc, (float *)dvc, heads, head_dim, scale, delta,
                                  st);
    if (status != HDT_OK) return status;
    {
        const long long total = (long long)B * heads * n_enc * chunks;
        HdtTimer tm("hdt_cross_scatter", st);
        hipLaunchKernelGGL(k_cross_scatter, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, l->cross_rank, n_enc, n_c,
                           heads, chunks, (const u32x4 *)dkc, (const u32x4 *)dvc, (u32x4 *)dk, (u32x4 *)dv, total);
    }
    HDT_HIP_TRY(hipGetLastError());
    return HDT_OK;
}

// ---- key lists cut into pieces ---------------------------------------------------------------------------
// How many pieces for this many heads: enough row tiles for a thousand workgroups (measured on 512 decoder rows x
// 8192 keys x 48 heads: forward kernel 201 us uncut, 91 in 4 pieces, 85 in 8, 82 in 16 where combining the pieces
// costs more than that gains), pieces of at least 8 entries, and none at all where the backward works on compact
// tensors (few keys, short lists).
int hdt_cross_pieces(const hdt_layout_t *l, int heads)
{
    if (!l->cross || l->compact || !l->cross_split_range[0] || heads <= 0) return 1;
    const long long tiles = (long long)l->s.batch * l->s.tr * heads;
    int pieces = 1;
    while (pieces < 8 && tiles * pieces < 1024 && l->cross_entries_max / (2 * pieces) >= 8) pieces *= 2;
    return pieces;
}

static size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

// the schedule with the lists cut: every row tile once per piece, partial results of rows_pad rows per piece
static HdtSchedule split_schedule(const hdt_layout_t *l, int pieces)
{
    HdtSchedule s = l->s;
    const int k = pieces == 2 ? 0 : (pieces == 4 ? 1 : 2);
    s.q_range = l->cross_split_range[k];
    s.tr = pieces * l->s.tr;
    s.n_pos = pieces * l->s.tr * l->s.bm;
    return s;  // n_own, tr_own keep the real rows
}

size_t hdt_cross_fwd_workspace_bytes(const hdt_layout_t *l, int heads, int head_dim)
{
    const int pieces = hdt_cross_pieces(l, heads);
    if (pieces == 1) return 0;
    const size_t rows = (size_t)l->s.batch * heads * pieces * l->s.tr * l->s.bm;
    return align256(rows * head_dim * 2) + align256(rows * sizeof(float));
}

size_t hdt_cross_dq_workspace_bytes(const hdt_layout_t *l, int heads, int head_dim)
{
    const int pieces = hdt_cross_pieces(l, heads);
    if (pieces == 1) return 0;
    return align256((size_t)l->s.batch * heads * pieces * l->s.tr * l->s.bm * head_dim * 2);
}

hdt_status_t hdt_cross_fwd_split(const hdt_layout_t *l, const void *q, const void *k, const void *v, void *o, float *lse,
                                 int heads, int head_dim, float scale, void *workspace, hipStream_t st)
{
    const int pieces = hdt_cross_pieces(l, heads);
    const HdtSchedule s = split_schedule(l, pieces);
    const size_t rows = (size_t)s.batch * heads * s.n_pos;
    char *w = static_cast<char *>(workspace);
    void *o_part = w;
    float *lse_part = reinterpret_cast<float *>(w + align256(rows * head_dim * 2));
    if (hdt_status_t status = hdt_launch_fwd_bf16(s, q, k, v, o_part, lse_part, heads, head_dim, scale, st)) return status;
    const int rows_pad = l->s.tr * l->s.bm;
    const long long total = (long long)l->s.batch * heads * l->s.n_pos * (head_dim / 8);
    HdtTimer tm("hdt_cross_combine_fwd", st);
    const dim3 grid((unsigned)((total + 255) / 256)), block(256);
#define COMBINE(DD, PP)                                                                                                  \
    hipLaunchKernelGGL((k_cross_combine_fwd<DD, PP>), grid, block, 0, st, (const u32x4 *)o_part, lse_part, (u32x4 *)o, lse, \
                       l->s.n_pos, rows_pad, total)
    if (head_dim == 64) {
        if (pieces == 2) COMBINE(64, 2); else if (pieces == 4) COMBINE(64, 4); else COMBINE(64, 8);
    } else {
        if (pieces == 2) COMBINE(128, 2); else if (pieces == 4) COMBINE(128, 4); else COMBINE(128, 8);
    }
#undef COMBINE
    HDT_HIP_TRY(hipGetLastError());
    return HDT_OK;
}

// Workspace: D of the decoder rows, then the pieces' parts of dQ.
hdt_status_t hdt_cross_bwd_split(const hdt_layout_t *l, const void *q, const void *k, const void *v, const void *o,
                                 const float *lse, const void *d_o, void *dq, void *dk, void *dv, int heads,
                                 int head_dim, float scale, void *workspace, hipStream_t st)
{
    const int pieces = hdt_cross_pieces(l, heads);
    const HdtSchedule s = split_schedule(l, pieces);
    const size_t d_bytes = hdt_bwd_row_scalars_bytes((size_t)l->s.batch * heads * (size_t)l->s.n_pos);
    char *w = static_cast<char *>(workspace);
    float *delta = reinterpret_cast<float *>(w);
    void *dq_part = w + d_bytes;
    // D is computed over the real rows (the D pass takes its row count from the first schedule's n_own)
    if (hdt_status_t status = hdt_launch_bwd_bf16(s, l->transposed->s, q, k, v, o, lse, d_o, dq_part, dk, dv, heads, head_dim,
                                                  scale, delta, st))
        return status;
    const int rows_pad = l->s.tr * l->s.bm;
    const long long total = (long long)l->s.batch * heads * l->s.n_pos * (head_dim / 8);
    HdtTimer tm("hdt_cross_sum_dq", st);
    const dim3 grid((unsigned)((total + 255) / 256)), block(256);
#define SUM_DQ(DD, PP) \
    hipLaunchKernelGGL((k_cross_sum_dq<DD, PP>), grid, block, 0, st, (const u32x4 *)dq_part, (u32x4 *)dq, l->s.n_pos, rows_pad, total)
    if (head_dim == 64) {
        if (pieces == 2) SUM_DQ(64, 2); else if (pieces == 4) SUM_DQ(64, 4); else SUM_DQ(64, 8);
    } else {
        if (pieces == 2) SUM_DQ(128, 2); else if (pieces == 4) SUM_DQ(128, 4); else SUM_DQ(128, 8);
    }
#undef SUM_DQ
    HDT_HIP_TRY(hipGetLastError());
    return HDT_OK;
}
