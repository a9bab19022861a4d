// hdt_build_layout: per-position level/parent ids -> block-sparse tile schedule, on the device.
//
// What is computed is fixed by the paper (Sec. 3.2: a position attends to parent, siblings and
// children; App. A.1, Alg. 1: sort keys by hierarchy level, partition into blocks, process a block
// only if its mask has a non-zero entry).  How it is computed is ours:
//   1. key order: stable counting sort by level with wave ballots (one workgroup per sample);
//   2. per anchor, the range of sorted slots its children occupy (integer atomic min/max);
//   3. candidate tiles per query tile: every allowed key of a row lies in one of <= 2 slot ranges
//      (its siblings = the children of its parent, and its own children) or is one of 2 single
//      slots (itself, its parent), so a row marks O(1) ranges instead of testing n keys.  For
//      documents laid out in pre-order the ranges are exact; for any other forest they are a
//      superset;
//   4. every candidate tile is then evaluated exactly, pair by pair (bitmap, pair count, 32x32
//      sub-block summary), and empty candidates are dropped, so the result never depends on
//      step 3 being tight;
//   5. compaction into lists by query tile and their transpose by key tile (prefix sums; all
//      orders are fixed by index, no ordering depends on atomics).
#include <limits.h>
#include <string.h>

#include <new>

#include "hdt_internal.h"

namespace {

constexpr int kSortThreads = 1024;
constexpr int kSortWaves = kSortThreads / 64;
constexpr int kBuckets = HDT_MAX_LEVELS + 1;  // levels 0..31, pads in the last bucket

__device__ __forceinline__ unsigned long long lanemask_lt()
{
    return (1ull << (threadIdx.x & 63)) - 1ull;
}

// ---- 1. validation + stable sort of positions by level ------------------------------------
__global__ __launch_bounds__(kSortThreads) void k_sort_by_level(const int32_t *__restrict__ level,
                                                                 const int32_t *__restrict__ parent, int n,
                                                                 int n_slots, int no_sort, int32_t *kperm,
                                                                 int32_t *slot, int32_t *cmin, int32_t *cmax,
                                                                 int32_t *err)
{
    const int b = blockIdx.x;
    level += (size_t)b * n;
    parent += (size_t)b * n;
    kperm += (size_t)b * n_slots;
    slot += (size_t)b * n;
    cmin += (size_t)b * n;
    cmax += (size_t)b * n;

    __shared__ volatile int s_cnt[kSortWaves][kBuckets];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;

    for (int i = tid; i < n; i += kSortThreads) {
        cmin[i] = INT_MAX;
        cmax[i] = -1;
    }
    for (int s = n + tid; s < n_slots; s += kSortThreads) kperm[s] = -1;
    for (int i = tid; i < kSortWaves * kBuckets; i += kSortThreads) (&s_cnt[0][0])[i] = 0;
    __syncthreads();

    // each wave owns a contiguous segment whose length is a multiple of 64
    const int seg = ((n + kSortWaves * 64 - 1) / (kSortWaves * 64)) * 64;
    const int begin = min(n, wave * seg), end = min(n, begin + seg);

    // pass A: validate, count positions per (wave, bucket)
    bool bad = false;
    for (int base = begin; base < end; base += 64) {
        const int i = base + lane;
        const bool in = i < end;
        int bucket = kBuckets - 1;
        if (in) {
            const int lv = level[i], p = parent[i];
            if (lv < -1 || lv >= HDT_MAX_LEVELS || p < -1 || p >= n || p == i || (lv < 0 && p != -1)) bad = true;
            if (lv >= 0 && lv < HDT_MAX_LEVELS) bucket = lv;
        }
        unsigned long long remaining = __ballot(in);
        while (remaining) {
            const int leader = __ffsll((long long)remaining) - 1;
            const int bk = __shfl(bucket, leader);
            const unsigned long long m = __ballot(in && bucket == bk);
            if (lane == 0) s_cnt[wave][bk] += __popcll(m);
            remaining &= ~m;
        }
    }
    if (__ballot(bad) && lane == 0) atomicOr(&err[0], 1);
    __syncthreads();

    // exclusive prefix over (bucket major, wave minor): first slot of every (wave, bucket)
    if (tid == 0) {
        int off = 0;
        for (int k = 0; k < kBuckets; k++)
            for (int w = 0; w < kSortWaves; w++) {
                const int c = s_cnt[w][k];
                s_cnt[w][k] = off;
                off += c;
            }
    }
    __syncthreads();

    // pass B: hand out slots in document order inside every bucket
    for (int base = begin; base < end; base += 64) {
        const int i = base + lane;
        const bool in = i < end;
        int bucket = kBuckets - 1;
        if (in) {
            const int lv = level[i];
            if (lv >= 0 && lv < HDT_MAX_LEVELS) bucket = lv;
        }
        int my_slot = i;
        unsigned long long remaining = __ballot(in);
        while (remaining) {
            const int leader = __ffsll((long long)remaining) - 1;
            const int bk = __shfl(bucket, leader);
            const bool mine = in && bucket == bk;
            const unsigned long long m = __ballot(mine);
            const int first = s_cnt[wave][bk];
            if (mine) my_slot = first + __popcll(m & lanemask_lt());
            __builtin_amdgcn_wave_barrier();
            if (lane == 0) s_cnt[wave][bk] = first + __popcll(m);
            __builtin_amdgcn_wave_barrier();
            remaining &= ~m;
        }
        if (in) {
            if (no_sort) my_slot = i;
            slot[i] = my_slot;
            kperm[my_slot] = i;
        }
    }
}

// ---- 2. slot range of every node's children ---------------------------------------------------
__global__ __launch_bounds__(256) void k_child_ranges(const int32_t *__restrict__ level,
                                                      const int32_t *__restrict__ parent,
                                                      const int32_t *__restrict__ slot, int n, int32_t *cmin,
                                                      int32_t *cmax, int32_t *err)
{
    const int b = blockIdx.y;
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const size_t o = (size_t)b * n;
    const int lv = level[o + i], p = parent[o + i];
    if (lv < 0 || p < 0 || p >= n) return;
    if (level[o + p] < 0) {  // a parent must be a real position
        atomicOr(&err[0], 1);
        return;
    }
    const int s = slot[o + i];
    atomicMin(&cmin[o + p], s);
    atomicMax(&cmax[o + p], s);
}

// ---- 3. candidate key tiles of every query tile -------------------------------------------------
__device__ __forceinline__ void mark_tiles(uint32_t *bits, int tlo, int thi)
{
    for (int w = tlo >> 5; w <= (thi >> 5); w++) {
        const int lo = max(tlo, w << 5) & 31, hi = min(thi, (w << 5) + 31) & 31;
        const uint32_t m = (hi == 31 ? 0xffffffffu : ((1u << (hi + 1)) - 1u)) & ~((1u << lo) - 1u);
        atomicOr(&bits[w], m);
    }
}

__global__ __launch_bounds__(128) void k_mark_candidates(const int32_t *__restrict__ level,
                                                         const int32_t *__restrict__ parent,
                                                         const int32_t *__restrict__ slot,
                                                         const int32_t *__restrict__ cmin,
                                                         const int32_t *__restrict__ cmax, int n, int bm, int bn,
                                                         int tr, int tc, int wc, int force_dense, uint32_t *cand,
                                                         int32_t *cand_cnt)
{
    extern __shared__ uint32_t s_bits[];
    __shared__ int s_total;
    const int I = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const size_t o = (size_t)b * n;
    for (int w = tid; w < wc; w += 128) s_bits[w] = 0;
    if (tid == 0) s_total = 0;
    __syncthreads();
    if (force_dense) {
        if (tid == 0) mark_tiles(s_bits, 0, tc - 1);
    } else if (tid < bm) {
        const int i = I * bm + tid;
        if (i < n && level[o + i] >= 0) {
            const int si = slot[o + i] / bn;
            mark_tiles(s_bits, si, si);  // itself
            const int p = parent[o + i];
            if (p >= 0 && p < n && level[o + p] >= 0) {
                const int sp = slot[o + p] / bn;
                mark_tiles(s_bits, sp, sp);  // its parent
                const int lo = cmin[o + p], hi = cmax[o + p];  // its siblings: children of the parent
                if (lo <= hi && lo >= 0 && hi < n) mark_tiles(s_bits, lo / bn, hi / bn);
            }
            const int lo = cmin[o + i], hi = cmax[o + i];  // its children
            if (lo <= hi && lo >= 0 && hi < n) mark_tiles(s_bits, lo / bn, hi / bn);
        }
    }
    __syncthreads();
    int local = 0;
    uint32_t *out = cand + ((size_t)b * tr + I) * wc;
    for (int w = tid; w < wc; w += 128) {
        const uint32_t v = s_bits[w];
        out[w] = v;
        local += __popc(v);
    }
    if (local) atomicAdd(&s_total, local);
    __syncthreads();
    if (tid == 0) cand_cnt[(size_t)b * tr + I] = s_total;
}

// ---- exclusive scan of a short int array by one workgroup ------------------------------------
__global__ __launch_bounds__(1024) void k_exclusive_scan(const int32_t *__restrict__ in, int32_t *out, int n,
                                                         int32_t *total_out)
{
    __shared__ int s_wave[16];
    __shared__ int s_carry;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    if (tid == 0) s_carry = 0;
    __syncthreads();
    for (int base = 0; base < n; base += 1024) {
        const int i = base + tid;
        const int v = i < n ? in[i] : 0;
        int x = v;  // inclusive scan inside the wave
        for (int d = 1; d < 64; d <<= 1) {
            const int y = __shfl_up(x, d);
            if (lane >= d) x += y;
        }
        if (lane == 63) s_wave[wave] = x;
        __syncthreads();
        int wave_off = 0;
        for (int w = 0; w < wave; w++) wave_off += s_wave[w];
        const int carry = s_carry;
        if (i < n) out[i] = carry + wave_off + x - v;
        __syncthreads();
        if (tid == 1023) s_carry = carry + wave_off + x;
        __syncthreads();
    }
    if (tid == 0) {
        out[n] = s_carry;
        if (total_out) *total_out = s_carry;
    }
}

// ---- 4. exact evaluation of every candidate tile ---------------------------------------------
// 4a: one wave per query tile lists its candidates: c_row[c] = query tile (global), c_col[c] = key tile
__global__ __launch_bounds__(64) void k_expand_candidates(const uint32_t *__restrict__ cand,
                                                          const int32_t *__restrict__ cand_ptr, int tr, int wc,
                                                          int64_t capacity, int32_t *c_row, int32_t *c_col)
{
    const int I = blockIdx.x, b = blockIdx.y, lane = threadIdx.x;
    const size_t row = (size_t)b * tr + I;
    const int cbase = cand_ptr[row];
    int n_cand = 0;
    for (int w0 = 0; w0 < wc; w0 += 2) {
        const int w = w0 + (lane >> 5), bit = lane & 31;
        const uint32_t word = w < wc ? cand[row * wc + w] : 0u;
        const bool is_cand = (word >> bit) & 1u;
        const unsigned long long cm = __ballot(is_cand);
        const int64_t c = (int64_t)cbase + n_cand + __popcll(cm & lanemask_lt());
        if (is_cand && c < capacity) {
            c_row[c] = (int32_t)row;
            c_col[c] = (w << 5) + bit;
        }
        n_cand += __popcll(cm);
    }
}

// 4b: one workgroup per candidate tile: pair-by-pair bitmap (row-major words for export and the
// fp32 path, and per 32x32 sub-block the 16 x 64-bit lane masks the MFMA kernels apply to their
// accumulator registers), pair count and sub-block summary.
__global__ __launch_bounds__(256) void k_tile_bitmaps(const int32_t *__restrict__ level,
                                                      const int32_t *__restrict__ parent,
                                                      const int32_t *__restrict__ kperm,
                                                      const int32_t *__restrict__ c_row,
                                                      const int32_t *__restrict__ c_col, int n, int n_slots,
                                                      int bm, int bn, int tr, uint32_t *bits,
                                                      unsigned long long *bits_rm, int32_t *c_cnt, uint32_t *c_sub)
{
    __shared__ int s_kpos[128], s_kpar[128];
    __shared__ uint32_t s_words[128 * 4];
    __shared__ int s_cnt;
    __shared__ unsigned int s_any, s_all;
    const int64_t c = blockIdx.x;
    const int tid = threadIdx.x;
    const int row = c_row[c], J = c_col[c];
    const int b = row / tr, I = row - b * tr;
    const size_t o = (size_t)b * n;
    const int wpr = bn >> 5;
    const int words = bm * wpr;
    const int nsub = (bm >> 5) * wpr;
    if (tid < bn) {
        const int s = J * bn + tid;
        int pos = s < n_slots ? kperm[(size_t)b * n_slots + s] : -1;
        int par = -1;
        if (pos >= 0 && pos < n && level[o + pos] >= 0)
            par = parent[o + pos];
        else
            pos = -1;
        s_kpos[tid] = pos;
        s_kpar[tid] = par;
    }
    if (tid == 0) {
        s_cnt = 0;
        s_any = 0;
        s_all = 0xffffu;
    }
    __syncthreads();
    for (int idx = tid; idx < words; idx += 256) {
        const int r = idx / wpr, wd = idx - r * wpr;
        const int i = I * bm + r;
        uint32_t out = 0;
        if (i < n && level[o + i] >= 0) {
            const int pi = parent[o + i];
            for (int cc = 0; cc < 32; cc++) {
                const int kj = s_kpos[wd * 32 + cc], kp = s_kpar[wd * 32 + cc];
                const bool ok = kj >= 0 && (kj == i || (pi >= 0 && pi == kp) || pi == kj || kp == i);
                out |= (uint32_t)ok << cc;
            }
        }
        bits[(size_t)c * words + idx] = out;
        s_words[idx] = out;
        const int sub = (r >> 5) * wpr + wd;
        if (out) {
            atomicAdd(&s_cnt, __popc(out));
            atomicOr(&s_any, 1u << sub);
        }
        if (out != 0xffffffffu) atomicAnd(&s_all, ~(1u << sub));
    }
    __syncthreads();
    // register-major masks: sub-block sb = rblk*wpr + cblk, accumulator register e, lane l:
    // row rblk*32 + l%32, column cblk*32 + (l/32)*4 + 8*(e/4) + e%4
    for (int idx = tid; idx < nsub * 16; idx += 256) {
        const int sb = idx >> 4, e = idx & 15;
        const int rblk = sb / wpr, cblk = sb - rblk * wpr;
        unsigned long long m = 0;
        for (int l = 0; l < 64; l++) {
            const uint32_t w = s_words[(rblk * 32 + (l & 31)) * wpr + cblk];
            const int bit = (l >> 5) * 4 + 8 * (e >> 2) + (e & 3);
            m |= (unsigned long long)((w >> bit) & 1u) << l;
        }
        bits_rm[(size_t)c * nsub * 16 + idx] = m;
    }
    if (tid == 0) {
        const unsigned int all = s_all & ((1u << nsub) - 1u);
        c_cnt[c] = s_cnt;
        c_sub[c] = s_any | (all << 16);
    }
}

// 4c: surviving tiles per query tile, and the per-sample totals
__global__ __launch_bounds__(64) void k_row_counts(const int32_t *__restrict__ cand_ptr,
                                                   const int32_t *__restrict__ c_cnt, int tr, int force_dense,
                                                   int64_t capacity, int32_t *row_cnt, unsigned long long *stats)
{
    const int I = blockIdx.x, b = blockIdx.y, lane = threadIdx.x;
    const size_t row = (size_t)b * tr + I;
    const int c0 = cand_ptr[row], c1 = cand_ptr[row + 1];
    int alive = 0;
    long long nnz = 0;
    for (int c = c0 + lane; c < c1 && c < capacity; c += 64) {
        const int cnt = c_cnt[c];
        if (cnt > 0 || force_dense) {
            alive++;
            nnz += cnt;
        }
    }
    for (int d = 32; d > 0; d >>= 1) {
        alive += __shfl_xor(alive, d);
        nnz += __shfl_xor(nnz, d);
    }
    if (lane == 0) {
        row_cnt[row] = alive;
        if (alive) {
            atomicAdd(&stats[2 * b], (unsigned long long)alive);
            atomicAdd(&stats[2 * b + 1], (unsigned long long)nnz);
        }
    }
}

// ---- 5a. lists by query tile -------------------------------------------------------------------
// One wave per query tile.  Rewrites `cand` in place to hold only the surviving tiles and
// fills `pre` with the number of surviving tiles in the words before each word.
__global__ __launch_bounds__(64) void k_compact_rows(uint32_t *cand, const int32_t *__restrict__ cand_ptr,
                                                     const int32_t *__restrict__ q_rowptr,
                                                     const int32_t *__restrict__ c_cnt,
                                                     const uint32_t *__restrict__ c_sub, int tr, int tc, int wc,
                                                     int force_dense, int64_t capacity, int32_t *pre,
                                                     int32_t *q_cols, uint32_t *q_sub, int32_t *q_bidx,
                                                     int32_t *k_cnt)
{
    const int I = blockIdx.x, b = blockIdx.y, lane = threadIdx.x;
    const size_t row = (size_t)b * tr + I;
    const int cbase = cand_ptr[row], tbase = q_rowptr[row];
    int n_cand = 0, n_alive = 0;
    for (int w0 = 0; w0 < wc; w0 += 2) {
        const int w = w0 + (lane >> 5), bit = lane & 31;
        const uint32_t word = w < wc ? cand[row * wc + w] : 0u;
        const bool is_cand = (word >> bit) & 1u;
        const unsigned long long cm = __ballot(is_cand);
        const int64_t c = (int64_t)cbase + n_cand + __popcll(cm & lanemask_lt());
        const bool alive = is_cand && c < capacity && (force_dense || c_cnt[c] > 0);
        const unsigned long long am = __ballot(alive);
        const int before = n_alive + __popcll(am & lanemask_lt());
        if (alive) {
            const int t = tbase + before;
            const int J = (w << 5) + bit;
            q_cols[t] = J;
            q_sub[t] = c_sub[c];
            q_bidx[t] = (int32_t)c;
            atomicAdd(&k_cnt[(size_t)b * tc + J], 1);
        }
        if (bit == 0 && w < wc) {
            pre[row * wc + w] = before;
            cand[row * wc + w] = (uint32_t)(am >> (lane & 32));
        }
        n_cand += __popcll(cm);
        n_alive += __popcll(am);
    }
}

// ---- 5b. transpose: lists by key tile, query tiles ascending --------------------------------
__global__ __launch_bounds__(64) void k_transpose(const uint32_t *__restrict__ alive,
                                                  const int32_t *__restrict__ pre,
                                                  const int32_t *__restrict__ q_rowptr,
                                                  const int32_t *__restrict__ k_colptr, int tr, int tc, int wc,
                                                  int32_t *k_rows, int32_t *k_tile)
{
    const int J = blockIdx.x * 64 + threadIdx.x, b = blockIdx.y;
    if (J >= tc) return;
    int e = k_colptr[(size_t)b * tc + J];
    const int w = J >> 5, bit = J & 31;
    for (int I = 0; I < tr; I++) {
        const size_t row = (size_t)b * tr + I;
        const uint32_t word = alive[row * wc + w];
        if ((word >> bit) & 1u) {
            k_rows[e] = I;
            k_tile[e] = q_rowptr[row] + pre[row * wc + w] + __popc(word & ((1u << bit) - 1u));
            e++;
        }
    }
}

// carve `bytes` (rounded up to 256) out of an arena
struct Carver {
    char *base;
    size_t off = 0;
    template <typename T>
    T *take(size_t count)
    {
        T *p = base ? reinterpret_cast<T *>(base + off) : nullptr;
        off += (count * sizeof(T) + 255) & ~(size_t)255;
        return p;
    }
};

struct Phase1 {
    int32_t *kperm, *slot, *cmin, *cmax, *cand_cnt, *cand_ptr, *row_cnt, *q_rowptr, *k_cnt, *k_colptr, *pre, *err;
    uint32_t *cand;
    int64_t *stats;
    size_t zero_begin, zero_end;  // byte range that must start at zero
    size_t bytes;
};

Phase1 carve_phase1(char *base, int B, int n, int n_slots, int tr, int tc, int wc)
{
    Carver c{base};
    Phase1 p;
    p.kperm = c.take<int32_t>((size_t)B * n_slots);
    p.slot = c.take<int32_t>((size_t)B * n);
    p.cmin = c.take<int32_t>((size_t)B * n);
    p.cmax = c.take<int32_t>((size_t)B * n);
    p.cand = c.take<uint32_t>((size_t)B * tr * wc);
    p.pre = c.take<int32_t>((size_t)B * tr * wc);
    p.cand_cnt = c.take<int32_t>((size_t)B * tr);
    p.cand_ptr = c.take<int32_t>((size_t)B * tr + 1);
    p.row_cnt = c.take<int32_t>((size_t)B * tr);
    p.q_rowptr = c.take<int32_t>((size_t)B * tr + 1);
    p.k_colptr = c.take<int32_t>((size_t)B * tc + 1);
    p.zero_begin = c.off;
    p.k_cnt = c.take<int32_t>((size_t)B * tc);
    p.stats = c.take<int64_t>((size_t)B * 2);
    p.err = c.take<int32_t>(4);
    p.zero_end = c.off;
    p.bytes = c.off;
    return p;
}

}  // namespace

extern "C" __attribute__((visibility("default"))) hdt_status_t hdt_build_layout(const int32_t *d_level, const int32_t *d_parent, int32_t batch,
                                         int32_t n_pos, const hdt_layout_opts_t *opts, void *stream,
                                         hdt_layout_t **out)
{
    if (!out) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_build_layout: out is NULL");
    *out = nullptr;
    if (batch < 0 || n_pos < 0) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_build_layout: negative size");
    if (n_pos > (1 << 22)) return hdt_fail(HDT_ERR_SHAPE, "hdt_build_layout: n_pos %d > 2^22", n_pos);
    int bm = 128, bn = 64, force_dense = 0, no_sort = 0;
    if (opts) {
        if (opts->tile_m) bm = opts->tile_m;
        if (opts->tile_n) bn = opts->tile_n;
        force_dense = opts->force_dense != 0;
        no_sort = opts->no_sort != 0;
    }
    if (bm < 32 || bm > 128 || bm % 32 || bn < 32 || bn > 128 || bn % 32)
        return hdt_fail(HDT_ERR_UNSUPPORTED, "hdt_build_layout: tile %dx%d (each side: 32, 64, 96 or 128)", bm, bn);
    const bool empty = batch == 0 || n_pos == 0;
    if (!empty && (!d_level || !d_parent)) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_build_layout: NULL id array");

    hdt_layout_t *L = new (std::nothrow) hdt_layout_t();
    if (!L) return hdt_fail(HDT_ERR_OOM, "hdt_build_layout: host allocation failed");
    L->magic = HDT_LAYOUT_MAGIC;
    L->arena = L->arena2 = nullptr;
    L->d_stats = nullptr;
    L->stats_cached = false;
    L->capacity = 0;
    L->device_bytes = 0;
    L->device = 0;
    HdtSchedule &s = L->s;
    memset(&s, 0, sizeof(s));
    s.batch = batch;
    s.n_pos = n_pos;
    s.bm = bm;
    s.bn = bn;
    s.wpr = bn / 32;
    s.tr = empty ? 0 : (n_pos + bm - 1) / bm;
    s.tc = empty ? 0 : (n_pos + bn - 1) / bn;
    s.n_slots = s.tc * bn;
    if (empty) {
        if (batch == 0) s.tr = s.tc = s.n_slots = 0;
        L->stats_cached = true;
        L->h_stats.assign((size_t)batch * 2, 0);
        *out = L;
        return HDT_OK;
    }
    if ((int64_t)batch * s.tr > (1 << 24) || (int64_t)batch * n_pos > (1LL << 30)) {
        delete L;
        return hdt_fail(HDT_ERR_SHAPE, "hdt_build_layout: batch * n_pos too large");
    }

    hipStream_t st = (hipStream_t)stream;
    const int B = batch, n = n_pos, tr = s.tr, tc = s.tc, wc = (tc + 31) / 32;
    hdt_status_t status = HDT_OK;
#define BUILD_TRY(expr)                                                                                  \
    do {                                                                                                 \
        hipError_t _e = (expr);                                                                          \
        if (_e != hipSuccess) {                                                                          \
            status = hdt_fail(_e == hipErrorOutOfMemory ? HDT_ERR_OOM : HDT_ERR_HIP, "%s: %s", #expr,  \
                              hipGetErrorString(_e));                                                    \
            goto fail;                                                                                   \
        }                                                                                                \
    } while (0)

    {
        (void)hipGetDevice(&L->device);
        Phase1 p = carve_phase1(nullptr, B, n, s.n_slots, tr, tc, wc);
        BUILD_TRY(hipMalloc(&L->arena, p.bytes));
        p = carve_phase1((char *)L->arena, B, n, s.n_slots, tr, tc, wc);
        L->device_bytes = (int64_t)p.bytes;
        BUILD_TRY(hipMemsetAsync((char *)L->arena + p.zero_begin, 0, p.zero_end - p.zero_begin, st));
        {
            HdtTimer t("hdt_layout_sort", st);
            hipLaunchKernelGGL(k_sort_by_level, dim3(B), dim3(kSortThreads), 0, st, d_level, d_parent, n, s.n_slots,
                               no_sort, p.kperm, p.slot, p.cmin, p.cmax, p.err);
        }
        {
            HdtTimer t("hdt_layout_child_ranges", st);
            hipLaunchKernelGGL(k_child_ranges, dim3((n + 255) / 256, B), dim3(256), 0, st, d_level, d_parent, p.slot, n,
                               p.cmin, p.cmax, p.err);
        }
        {
            HdtTimer t("hdt_layout_mark", st);
            hipLaunchKernelGGL(k_mark_candidates, dim3(tr, B), dim3(128), (size_t)wc * sizeof(uint32_t), st, d_level,
                               d_parent, p.slot, p.cmin, p.cmax, n, bm, bn, tr, tc, wc, force_dense, p.cand,
                               p.cand_cnt);
        }
        {
            HdtTimer t("hdt_layout_scan", st);
            hipLaunchKernelGGL(k_exclusive_scan, dim3(1), dim3(1024), 0, st, p.cand_cnt, p.cand_ptr, B * tr, p.err + 1);
        }
        BUILD_TRY(hipGetLastError());
        int32_t h_err[2] = {0, 0};
        BUILD_TRY(hipMemcpyAsync(h_err, p.err, sizeof(h_err), hipMemcpyDeviceToHost, st));
        BUILD_TRY(hipStreamSynchronize(st));
        if (h_err[0]) {
            status = hdt_fail(HDT_ERR_HIERARCHY,
                              "hdt_build_layout: level/parent arrays are not a valid hierarchy (level outside "
                              "[-1, %d), parent outside [-1, n_pos), self-parent, pad with a parent, or pad parent)",
                              HDT_MAX_LEVELS);
            goto fail;
        }
        const int64_t cap = h_err[1];
        L->capacity = cap;
        const size_t words = (size_t)bm * s.wpr;
        Carver c2{nullptr};
        for (int pass = 0; pass < 2; pass++) {
            c2.off = 0;
            int32_t *q_cols = c2.take<int32_t>((size_t)cap);
            uint32_t *q_sub = c2.take<uint32_t>((size_t)cap);
            int32_t *q_bidx = c2.take<int32_t>((size_t)cap);
            int32_t *c_col = c2.take<int32_t>((size_t)cap);
            int32_t *c_cnt = c2.take<int32_t>((size_t)cap);
            uint32_t *c_sub = c2.take<uint32_t>((size_t)cap);
            int32_t *k_rows = c2.take<int32_t>((size_t)cap);
            int32_t *k_tile = c2.take<int32_t>((size_t)cap);
            uint32_t *bits = c2.take<uint32_t>((size_t)cap * words);
            unsigned long long *bits_rm = c2.take<unsigned long long>((size_t)cap * (bm / 32) * s.wpr * 16);
            int32_t *c_row = c2.take<int32_t>((size_t)cap);
            if (pass == 0) {
                if (cap > 0) BUILD_TRY(hipMalloc(&L->arena2, c2.off));
                c2.base = (char *)L->arena2;
                L->device_bytes += cap > 0 ? (int64_t)c2.off : 0;
                continue;
            }
            s.kperm = p.kperm;
            s.q_rowptr = p.q_rowptr;
            s.q_cols = q_cols;
            s.q_sub = q_sub;
            s.q_bidx = q_bidx;
            s.bits = bits;
            s.bits_rm = bits_rm;
            s.k_colptr = p.k_colptr;
            s.k_rows = k_rows;
            s.k_tile = k_tile;
            L->d_stats = p.stats;
            {
                HdtTimer t("hdt_layout_expand", st);
                hipLaunchKernelGGL(k_expand_candidates, dim3(tr, B), dim3(64), 0, st, p.cand, p.cand_ptr, tr, wc, cap,
                                   c_row, c_col);
            }
            if (cap > 0) {
                HdtTimer t("hdt_layout_tile_bitmaps", st);
                hipLaunchKernelGGL(k_tile_bitmaps, dim3((unsigned)cap), dim3(256), 0, st, d_level, d_parent, p.kperm,
                                   c_row, c_col, n, s.n_slots, bm, bn, tr, bits, bits_rm, c_cnt, c_sub);
            }
            {
                HdtTimer t("hdt_layout_row_counts", st);
                hipLaunchKernelGGL(k_row_counts, dim3(tr, B), dim3(64), 0, st, p.cand_ptr, c_cnt, tr, force_dense, cap,
                                   p.row_cnt, (unsigned long long *)p.stats);
            }
            {
                HdtTimer t("hdt_layout_scan", st);
                hipLaunchKernelGGL(k_exclusive_scan, dim3(1), dim3(1024), 0, st, p.row_cnt, p.q_rowptr, B * tr,
                                   (int32_t *)nullptr);
            }
            {
                HdtTimer t("hdt_layout_compact", st);
                hipLaunchKernelGGL(k_compact_rows, dim3(tr, B), dim3(64), 0, st, p.cand, p.cand_ptr, p.q_rowptr, c_cnt,
                                   c_sub, tr, tc, wc, force_dense, cap, p.pre, q_cols, q_sub, q_bidx, p.k_cnt);
            }
            {
                HdtTimer t("hdt_layout_scan", st);
                hipLaunchKernelGGL(k_exclusive_scan, dim3(1), dim3(1024), 0, st, p.k_cnt, p.k_colptr, B * tc,
                                   (int32_t *)nullptr);
            }
            {
                HdtTimer t("hdt_layout_transpose", st);
                hipLaunchKernelGGL(k_transpose, dim3((tc + 63) / 64, B), dim3(64), 0, st, p.cand, p.pre, p.q_rowptr,
                                   p.k_colptr, tr, tc, wc, k_rows, k_tile);
            }
            BUILD_TRY(hipGetLastError());
        }
    }
    *out = L;
    return HDT_OK;
fail:
    if (L->arena) (void)hipFree(L->arena);
    if (L->arena2) (void)hipFree(L->arena2);
    L->magic = 0;
    delete L;
    return status;
#undef BUILD_TRY
}
