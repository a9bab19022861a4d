// hdt_build_layout: per-position level/parent ids -> block-sparse tile schedule, on the device.
//
// What is computed is fixed by the paper (Sec. 3.2: a position attends to parent, siblings and
// children; App. A.1, Alg. 1: sort keys by hierarchy level, partition into blocks, process a block
// only if its mask has a non-zero entry).  How it is computed is ours.  Three kernels:
//
//  front (one workgroup per sample)
//   1. key order: stable counting sort by level with wave ballots;
//   2. per anchor, the range of sorted slots its children occupy (integer atomic min/max, one
//      pair of atomics per run of consecutive children);
//   3. candidate tiles per query tile: every allowed key of a row lies in one of <= 2 slot ranges
//      (its siblings = the children of its parent, and its own children) or is one of 2 single
//      slots (itself, its parent), so a row marks O(1) ranges instead of testing n keys.  For
//      documents laid out in pre-order the ranges are exact; for any other forest they are a
//      superset;
//   4. prefix sum of the candidate counts, a slice of the per-tile arrays reserved with one atomic
//      add per sample, and the key tile of every candidate written out: these ARE the tile lists;
//  bitmaps (grid-stride over candidates)
//   5. every candidate tile is evaluated exactly, pair by pair (bitmap, pair count, 32x32
//      sub-block summary), so the result never depends on step 3 being tight.  A candidate without
//      any allowed pair keeps its list entry with an all-zero summary, which every kernel skips;
//      it is not counted as a tile and hdt_layout_export leaves it out.
//
// The per-tile arrays are sized before the number of candidates is known (a heuristic, raised by
// what earlier builds needed); both kernels check the capacity.  The front kernel reports the count
// (and whether the hierarchy was valid) through one word of pinned host memory as soon as it is
// known; the host waits for that word only, not for the stream, and repeats the build with the exact
// size in the rare case the guess was too small.
// Device memory comes from a small cache of earlier layouts' buffers.
#include <limits.h>
#include <string.h>

#include <algorithm>
#include <chrono>
#include <mutex>
#include <new>
#include <vector>

#include "hdt_internal.h"

namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / 64;
constexpr int kBuckets = HDT_MAX_LEVELS + 1;  // levels 0..31, pads in the last bucket
constexpr int kSortChunk = 8;                 // positions per lane loaded ahead of the ballot loops

enum { CNT_ERR = 0, CNT_CAND = 1, CNT_TILES = 2, CNT_ARRIVED = 3 };

// What the front kernel reports to the host through pinned host memory: one 64-bit word
// [63:40] ticket of the build, [39] hierarchy error, [31:0] candidate tiles needed.
__host__ __device__ inline unsigned long long report_word(uint32_t ticket, int err, uint32_t need)
{
    return ((unsigned long long)(ticket & 0xffffffu) << 40) | ((unsigned long long)(err != 0) << 39) | need;
}

__device__ __forceinline__ unsigned long long lanemask_lt() { return (1ull << (threadIdx.x & 63)) - 1ull; }

__device__ __forceinline__ int wave_sum(int x)
{
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) x += __shfl_xor(x, d);
    return x;
}

// exclusive scan, in place, of data[0..n) by the whole workgroup; returns the total to every thread
__device__ int block_scan_inplace(int32_t *data, int n, int *s_wave /*[kWaves + 1]*/)
{
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    int carry = 0;
    for (int base = 0; base < n; base += kThreads) {
        const int i = base + tid;
        const int v = i < n ? data[i] : 0;
        int x = v;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int y = __shfl_up(x, d);
            if (lane >= d) x += y;
        }
        if (lane == 63) s_wave[wave] = x;
        __syncthreads();
        int off = 0, tot = 0;
        for (int w = 0; w < kWaves; w++) {
            const int sw = s_wave[w];
            if (w < wave) off += sw;
            tot += sw;
        }
        if (i < n) data[i] = carry + off + x - v;
        carry += tot;
        __syncthreads();
    }
    return carry;
}

__device__ __forceinline__ void mark_tiles(uint32_t *bits, int tlo, int thi)
{
    for (int w = tlo >> 5; w <= (thi >> 5); w++) {
        const int lo = max(tlo, w << 5) & 31, hi = min(thi, (w << 5) + 31) & 31;
        const uint32_t m = (hi == 31 ? 0xffffffffu : ((1u << (hi + 1)) - 1u)) & ~((1u << lo) - 1u);
        atomicOr(&bits[w], m);
    }
}

struct FrontArgs {
    const int32_t *level, *parent;
    int n, n_slots, bm, bn, tr, tc, wc, force_dense, no_sort;
    int64_t capacity;
    int32_t *kperm, *slot, *cmin, *cmax;
    uint32_t *cand;     // [B][tr][wc]
    int32_t *cand_ptr;  // [B][tr+1]: becomes the lists' row pointer
    int32_t *c_row, *q_cols;
    int32_t *counters;
    unsigned long long *report;  // pinned host memory, written once by the last workgroup to get there
    uint32_t ticket;
};

// ---- front: sort, child ranges, candidates ---------------------------------------------------
__global__ __launch_bounds__(kThreads) void k_layout_front(FrontArgs a)
{
    extern __shared__ uint32_t s_bitmaps[];  // [kWaves][wc]
    __shared__ volatile int s_cnt[kWaves][kBuckets];
    __shared__ int s_wave[kWaves + 1];
    __shared__ int s_base;
    const int b = blockIdx.x, n = a.n;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int32_t *level = a.level + (size_t)b * n, *parent = a.parent + (size_t)b * n;
    int32_t *kperm = a.kperm + (size_t)b * a.n_slots, *slot = a.slot + (size_t)b * n;
    int32_t *cmin = a.cmin + (size_t)b * n, *cmax = a.cmax + (size_t)b * n;

    for (int i = tid; i < n; i += kThreads) {
        cmin[i] = INT_MAX;
        cmax[i] = -1;
    }
    for (int s = n + tid; s < a.n_slots; s += kThreads) kperm[s] = -1;
    for (int i = tid; i < kWaves * kBuckets; i += kThreads) (&s_cnt[0][0])[i] = 0;
    __syncthreads();

    // 1. stable sort by level.  Each wave owns a contiguous segment (a multiple of 64 positions); lane k
    // of a wave keeps the wave's running count of bucket k in a register.
    const int seg = ((n + kWaves * 64 - 1) / (kWaves * 64)) * 64;
    const int begin = min(n, wave * seg), end = min(n, begin + seg);
    bool bad = false;
    int mycnt = 0;
    for (int base = begin; base < end; base += 64 * kSortChunk) {  // pass A: validate and count
        int lv[kSortChunk], pr[kSortChunk];
#pragma unroll
        for (int u = 0; u < kSortChunk; u++) {
            const int i = base + u * 64 + lane;
            lv[u] = i < end ? level[i] : -1;
            pr[u] = i < end ? parent[i] : -1;
        }
#pragma unroll
        for (int u = 0; u < kSortChunk; u++) {
            const int i = base + u * 64 + lane;
            const bool in = i < end;
            int bucket = kBuckets - 1;
            if (in) {
                const int l = lv[u], p = pr[u];
                if (l < -1 || l >= HDT_MAX_LEVELS || p < -1 || p >= n || p == i || (l < 0 && p != -1)) bad = true;
                if (l >= 0 && l < HDT_MAX_LEVELS) bucket = l;
            }
            unsigned long long remaining = __ballot(in);
            while (remaining) {
                const int leader = __ffsll((long long)remaining) - 1;
                const int bk = __builtin_amdgcn_readlane(bucket, leader);
                const unsigned long long m = __ballot(in && bucket == bk);
                if (lane == bk) mycnt += __popcll(m);
                remaining &= ~m;
            }
        }
    }
    if (__ballot(bad) && lane == 0) atomicOr(&a.counters[CNT_ERR], 1);
    if (lane < kBuckets) s_cnt[wave][lane] = mycnt;
    __syncthreads();
    if (wave == 0) {  // first slot of every (bucket, wave): bucket major, wave minor; lane k scans bucket k
        int tot = 0, pre[kWaves];
        if (lane < kBuckets) {
#pragma unroll
            for (int w = 0; w < kWaves; w++) {
                pre[w] = tot;
                tot += s_cnt[w][lane];
            }
        }
        int incl = tot;  // inclusive scan of the bucket totals over lanes
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int y = __shfl_up(incl, d);
            if (lane >= d) incl += y;
        }
        if (lane < kBuckets) {
#pragma unroll
            for (int w = 0; w < kWaves; w++) s_cnt[w][lane] = incl - tot + pre[w];
        }
    }
    __syncthreads();
    int mybase = lane < kBuckets ? s_cnt[wave][lane] : 0;
    for (int base = begin; base < end; base += 64 * kSortChunk) {  // pass B: hand out slots in document order
        int lv[kSortChunk];
#pragma unroll
        for (int u = 0; u < kSortChunk; u++) {
            const int i = base + u * 64 + lane;
            lv[u] = i < end ? level[i] : -1;
        }
#pragma unroll
        for (int u = 0; u < kSortChunk; u++) {
            const int i = base + u * 64 + lane;
            const bool in = i < end;
            int bucket = kBuckets - 1;
            if (in && lv[u] >= 0 && lv[u] < HDT_MAX_LEVELS) bucket = lv[u];
            int my_slot = i;
            unsigned long long remaining = __ballot(in);
            while (remaining) {
                const int leader = __ffsll((long long)remaining) - 1;
                const int bk = __builtin_amdgcn_readlane(bucket, leader);
                const bool mine = in && bucket == bk;
                const unsigned long long m = __ballot(mine);
                const int first = __builtin_amdgcn_readlane(mybase, bk);
                if (mine) my_slot = first + __popcll(m & lanemask_lt());
                if (lane == bk) mybase += __popcll(m);
                remaining &= ~m;
            }
            if (in) {
                if (a.no_sort) my_slot = i;
                slot[i] = my_slot;
                kperm[my_slot] = i;
            }
        }
    }
    __threadfence_block();
    __syncthreads();

    // 2. slot range of every node's children.  Consecutive positions with the same parent and
    // consecutive slots (the tokens of a sentence, for one) form a run whose minimum and maximum are its
    // first and last slot: one atomic each per run.
    for (int base = 0; base < n; base += kThreads) {
        const int i = base + tid;
        int p = -1, sl = -1;
        bool valid = false;
        if (i < n) {
            const int l = level[i];
            p = parent[i];
            valid = l >= 0 && p >= 0 && p < n;
            if (valid && level[p] < 0) {  // a parent must be a real position
                atomicOr(&a.counters[CNT_ERR], 1);
                valid = false;
            }
            if (valid) sl = slot[i];
        }
        const int p_prev = __shfl_up(p, 1), s_prev = __shfl_up(sl, 1);
        const bool v_prev = __shfl_up((int)valid, 1) != 0;
        const bool head = lane == 0 || !v_prev || p_prev != p || s_prev + 1 != sl;
        const bool next_head = __shfl_down((int)(head || !valid), 1) != 0;  // lane+1 starts a new run (or is invalid)
        const bool tail = lane == 63 || next_head;
        if (valid && head) atomicMin(&cmin[p], sl);
        if (valid && tail) atomicMax(&cmax[p], sl);
    }
    __threadfence_block();
    __syncthreads();

    // 3. candidate key tiles of every query tile: one wave per query tile, a bitmap per wave in LDS
    const int bm = a.bm, bn = a.bn, tr = a.tr, tc = a.tc, wc = a.wc;
    uint32_t *wbits = s_bitmaps + (size_t)wave * wc;
    int32_t *cand_ptr = a.cand_ptr + (size_t)b * (tr + 1);
    for (int I = wave; I < tr; I += kWaves) {
        for (int w = lane; w < wc; w += 64) wbits[w] = 0;
        __builtin_amdgcn_wave_barrier();
        if (a.force_dense) {
            if (lane == 0) mark_tiles(wbits, 0, tc - 1);
        } else {
            // rows lane and lane + 64 of the tile; all loads of one dependency level are issued together
            int i2[2], sl2[2], p2[2], lo_c[2], hi_c[2];
            bool ok[2];
#pragma unroll
            for (int u = 0; u < 2; u++) {
                const int rr = lane + 64 * u;
                i2[u] = I * bm + rr;
                ok[u] = rr < bm && i2[u] < n && level[min(i2[u], n - 1)] >= 0;
                const int ii = ok[u] ? i2[u] : 0;
                sl2[u] = slot[ii];
                p2[u] = parent[ii];
                lo_c[u] = cmin[ii];
                hi_c[u] = cmax[ii];
            }
            int sp2[2], lo_s[2], hi_s[2];
            bool okp[2];
#pragma unroll
            for (int u = 0; u < 2; u++) {
                okp[u] = ok[u] && p2[u] >= 0 && p2[u] < n;
                const int pp = okp[u] ? p2[u] : 0;
                okp[u] = okp[u] && level[pp] >= 0;
                sp2[u] = slot[pp];
                lo_s[u] = cmin[pp];
                hi_s[u] = cmax[pp];
            }
#pragma unroll
            for (int u = 0; u < 2; u++) {
                if (!ok[u]) continue;
                mark_tiles(wbits, sl2[u] / bn, sl2[u] / bn);  // itself
                if (okp[u]) {
                    mark_tiles(wbits, sp2[u] / bn, sp2[u] / bn);  // its parent
                    if (lo_s[u] <= hi_s[u] && lo_s[u] >= 0 && hi_s[u] < n)
                        mark_tiles(wbits, lo_s[u] / bn, hi_s[u] / bn);  // its siblings: the children of its parent
                }
                if (lo_c[u] <= hi_c[u] && lo_c[u] >= 0 && hi_c[u] < n)
                    mark_tiles(wbits, lo_c[u] / bn, hi_c[u] / bn);  // its children
            }
        }
        __builtin_amdgcn_wave_barrier();
        int cnt = 0;
        uint32_t *out = a.cand + ((size_t)b * tr + I) * wc;
        for (int w = lane; w < wc; w += 64) {
            const uint32_t v = wbits[w];
            out[w] = v;
            cnt += __popc(v);
        }
        cnt = wave_sum(cnt);
        if (lane == 0) cand_ptr[I] = cnt;
        __builtin_amdgcn_wave_barrier();
    }
    __threadfence();  // device scope: this workgroup's error flags have reached the counters
    __syncthreads();

    // 4. prefix sum, reserve this sample's slice of the candidate arrays, list the candidates
    const int total = block_scan_inplace(cand_ptr, tr, s_wave);
    if (tid == 0) {
        s_base = atomicAdd(&a.counters[CNT_CAND], total);
        // the last workgroup to get here knows the final counters: it tells the host, which is waiting
        // for exactly this word, while the lists and the bitmaps are still being written
        __threadfence();
        if (atomicAdd(&a.counters[CNT_ARRIVED], 1) == (int)gridDim.x - 1) {
            __threadfence();
            const int err = __hip_atomic_load(&a.counters[CNT_ERR], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const int need = __hip_atomic_load(&a.counters[CNT_CAND], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(a.report, report_word(a.ticket, err, (uint32_t)need), __ATOMIC_RELEASE,
                               __HIP_MEMORY_SCOPE_SYSTEM);
        }
    }
    __syncthreads();
    const int gbase = s_base;
    for (int I = tid; I < tr; I += kThreads) cand_ptr[I] += gbase;
    if (tid == 0) cand_ptr[tr] = gbase + total;
    __threadfence_block();
    __syncthreads();
    for (int I = wave; I < tr; I += kWaves) {
        const size_t row = (size_t)b * tr + I;
        const int cbase = cand_ptr[I];
        int n_cand = 0;
        for (int w0 = 0; w0 < wc; w0 += 2) {
            const int w = w0 + (lane >> 5), bit = lane & 31;
            const uint32_t word = w < wc ? a.cand[row * wc + w] : 0u;
            const bool is_cand = (word >> bit) & 1u;
            const unsigned long long cm = __ballot(is_cand);
            const int64_t c = (int64_t)cbase + n_cand + __popcll(cm & lanemask_lt());
            if (is_cand && c < a.capacity) {
                a.c_row[c] = (int32_t)row;
                a.q_cols[c] = (w << 5) + bit;
            }
            n_cand += __popcll(cm);
        }
    }
}

// ---- bitmaps: exact evaluation of every candidate tile ------------------------------------------
// One candidate per workgroup iteration: pair-by-pair bitmap (row-major words for export and the
// fp32 path, and per 32x32 sub-block the 16 x 64-bit lane masks the MFMA kernels apply to their
// accumulator registers), pair count and sub-block summary.
__global__ __launch_bounds__(256) void k_tile_bitmaps(const int32_t *__restrict__ level,
                                                      const int32_t *__restrict__ parent,
                                                      const int32_t *__restrict__ kperm,
                                                      const int32_t *__restrict__ c_row,
                                                      const int32_t *__restrict__ c_col,
                                                      const int32_t *__restrict__ counters, int64_t capacity,
                                                      int n, int n_slots, int bm, int bn, int tr, uint32_t *bits,
                                                      unsigned long long *bits_rm, int32_t *c_cnt, uint32_t *c_sub)
{
    __shared__ int s_kpos[128], s_kpar[128];
    __shared__ uint32_t s_words[128 * 4];
    __shared__ int s_cnt;
    __shared__ unsigned int s_any, s_all;
    const int tid = threadIdx.x;
    const int wpr = bn >> 5;
    const int words = bm * wpr;
    const int nsub = (bm >> 5) * wpr;
    const int64_t total = min((int64_t)counters[CNT_CAND], capacity);
    for (int64_t c = blockIdx.x; c < total; c += gridDim.x) {
        const int row = c_row[c], J = c_col[c];
        const int b = row / tr, I = row - b * tr;
        const size_t o = (size_t)b * n;
        __syncthreads();  // the previous candidate's LDS words are no longer read
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
}

// ---- device memory: a small cache of buffers of destroyed layouts ------------------------------
struct CachedBlock {
    void *ptr;
    size_t bytes;
    int device;
};
std::mutex g_pool_mutex;
std::vector<CachedBlock> g_pool;
constexpr size_t kPoolMaxBlocks = 16;
constexpr size_t kPoolMaxBytes = (size_t)1 << 30;
int64_t g_capacity_hint = 0;  // candidates the last build needed

hipError_t pool_alloc(void **out, size_t bytes, size_t *got)
{
    int dev = 0;
    (void)hipGetDevice(&dev);
    {
        std::lock_guard<std::mutex> lk(g_pool_mutex);
        int best = -1;
        for (size_t i = 0; i < g_pool.size(); i++)
            if (g_pool[i].device == dev && g_pool[i].bytes >= bytes && g_pool[i].bytes <= 2 * bytes + (1 << 20) &&
                (best < 0 || g_pool[i].bytes < g_pool[best].bytes))
                best = (int)i;
        if (best >= 0) {
            *out = g_pool[best].ptr;
            *got = g_pool[best].bytes;
            g_pool.erase(g_pool.begin() + best);
            return hipSuccess;
        }
    }
    *got = bytes;
    return hipMalloc(out, bytes);
}

void pool_free(void *ptr, size_t bytes, int device)
{
    if (!ptr) return;
    {
        std::lock_guard<std::mutex> lk(g_pool_mutex);
        size_t held = 0;
        for (auto &b : g_pool) held += b.bytes;
        if (g_pool.size() < kPoolMaxBlocks && held + bytes <= kPoolMaxBytes) {
            g_pool.push_back({ptr, bytes, device});
            return;
        }
    }
    (void)hipFree(ptr);
}

// carve buffers (each rounded up to 256 bytes) out of an arena
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
    int32_t *kperm, *slot, *cmin, *cmax, *cand_ptr, *counters;
    uint32_t *cand;
    int64_t *stats;
    size_t zero_begin, zero_end;  // byte range that must start at zero (also what the host reads back)
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
    p.cand_ptr = c.take<int32_t>((size_t)B * (tr + 1));
    p.zero_begin = c.off;
    p.counters = c.take<int32_t>(64);  // 256 bytes, so that stats follows immediately
    p.stats = c.take<int64_t>((size_t)B * 2);
    p.zero_end = c.off;
    p.bytes = c.off;
    return p;
}

struct Phase2 {
    int32_t *q_cols, *c_row, *c_cnt;
    uint32_t *q_sub, *bits;
    unsigned long long *bits_rm;
    size_t bytes;
};

Phase2 carve_phase2(char *base, int64_t cap, int bm, int bn)
{
    Carver c{base};
    Phase2 p;
    const size_t n = (size_t)cap, words = (size_t)bm * (bn / 32), nsub = (size_t)(bm / 32) * (bn / 32);
    p.q_cols = c.take<int32_t>(n);
    p.q_sub = c.take<uint32_t>(n);
    p.c_row = c.take<int32_t>(n);
    p.c_cnt = c.take<int32_t>(n);
    p.bits = c.take<uint32_t>(n * words);
    p.bits_rm = c.take<unsigned long long>(n * nsub * 16);
    p.bytes = c.off;
    return p;
}

// ---- the build's report from the device: 64 words of pinned host memory, one per build in flight ----
constexpr int kReportSlots = 64;
unsigned long long *g_reports = nullptr;  // never freed: a kernel may still write to it at exit
uint32_t g_ticket = 0;

unsigned long long *report_slot(uint32_t *ticket)
{
    std::lock_guard<std::mutex> lk(g_pool_mutex);
    if (!g_reports) {
        void *ptr = nullptr;
        if (hipHostMalloc(&ptr, kReportSlots * 64, hipHostMallocPortable | hipHostMallocMapped) != hipSuccess) {
            (void)hipGetLastError();
            return nullptr;
        }
        memset(ptr, 0, kReportSlots * 64);
        g_reports = static_cast<unsigned long long *>(ptr);
    }
    g_ticket = (g_ticket + 1) & 0xffffffu;
    if (g_ticket == 0) g_ticket = 1;
    *ticket = g_ticket;
    return g_reports + (size_t)(g_ticket % kReportSlots) * 8;  // one 64-byte line per slot
}

// polls the word until it carries this build's ticket; false after 10 s without it
bool wait_for_report(const unsigned long long *slot, uint32_t ticket, unsigned long long *word)
{
    const auto t0 = std::chrono::steady_clock::now();
    for (uint64_t spins = 0;; spins++) {
        const unsigned long long w = __atomic_load_n(slot, __ATOMIC_ACQUIRE);
        if ((uint32_t)(w >> 40) == ticket) {
            *word = w;
            return true;
        }
        if ((spins & 0x3ff) == 0x3ff && std::chrono::steady_clock::now() - t0 > std::chrono::seconds(10)) return false;
        __builtin_ia32_pause();
    }
}

}  // namespace

void hdt_layout_release(hdt_layout_t *L)
{
    pool_free(L->arena, L->arena_bytes, L->device);
    pool_free(L->arena2, L->arena2_bytes, L->device);
    L->arena = L->arena2 = nullptr;
}

// Surviving tiles and allowed pairs per sample, summed on the host from the query tile and the pair
// count of every list entry (two adjacent device arrays): cheaper than thousands of device atomics on
// a handful of addresses, and only paid by callers that ask.
hdt_status_t hdt_layout_stats(const hdt_layout_t *L)
{
    static std::mutex stats_mutex;
    std::lock_guard<std::mutex> lk(stats_mutex);
    if (L->stats_ready) return HDT_OK;
    const int64_t E = L->n_entries;
    std::vector<int32_t> row((size_t)E), cnt((size_t)E);
    int dev = 0;
    HDT_HIP_TRY(hipGetDevice(&dev));
    if (dev != L->device) HDT_HIP_TRY(hipSetDevice(L->device));
    hipError_t e = hipDeviceSynchronize();
    if (e == hipSuccess && E > 0) e = hipMemcpy(row.data(), L->d_row, sizeof(int32_t) * E, hipMemcpyDeviceToHost);
    if (e == hipSuccess && E > 0) e = hipMemcpy(cnt.data(), L->d_cnt, sizeof(int32_t) * E, hipMemcpyDeviceToHost);
    if (dev != L->device) (void)hipSetDevice(dev);
    if (e != hipSuccess) return hdt_fail(HDT_ERR_HIP, "hdt_layout_stats: %s", hipGetErrorString(e));
    std::fill(L->h_stats.begin(), L->h_stats.end(), 0);
    const int B = L->s.batch, tr = L->s.tr;
    for (int64_t c = 0; c < E; c++) {
        const int b = row[c] / tr;
        if (b < 0 || b >= B) continue;
        if (cnt[c] > 0 || L->force_dense) {
            L->h_stats[2 * b] += 1;
            L->h_stats[2 * b + 1] += cnt[c];
        }
    }
    L->stats_ready = true;
    return HDT_OK;
}

extern "C" __attribute__((visibility("default"))) hdt_status_t hdt_release_cached_memory(void)
{
    std::vector<CachedBlock> blocks;
    {
        std::lock_guard<std::mutex> lk(g_pool_mutex);
        blocks.swap(g_pool);
    }
    hipError_t e = hipSuccess;
    for (auto &b : blocks) {
        hipError_t e2 = hipFree(b.ptr);
        if (e == hipSuccess) e = e2;
    }
    if (e != hipSuccess) return hdt_fail(HDT_ERR_HIP, "hipFree: %s", hipGetErrorString(e));
    return HDT_OK;
}

extern "C" __attribute__((visibility("default"))) hdt_status_t hdt_build_layout(const int32_t *d_level,
                                                                                 const int32_t *d_parent,
                                                                                 int32_t batch, int32_t n_pos,
                                                                                 const hdt_layout_opts_t *opts,
                                                                                 void *stream, hdt_layout_t **out)
{
    if (!out) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_build_layout: out is NULL");
    *out = nullptr;
    if (batch < 0 || n_pos < 0) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_build_layout: negative size");
    if (n_pos > (1 << 19)) return hdt_fail(HDT_ERR_SHAPE, "hdt_build_layout: n_pos %d > 2^19", n_pos);
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
    L->arena_bytes = L->arena2_bytes = 0;
    L->capacity = 0;
    L->d_cnt = nullptr;
    L->d_row = nullptr;
    L->n_entries = 0;
    L->stats_ready = false;
    L->force_dense = force_dense;
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
    L->h_stats.assign((size_t)batch * 2, 0);
    if (empty) {
        L->stats_ready = true;
        *out = L;
        return HDT_OK;
    }
    if ((int64_t)batch * n_pos > (1LL << 30) || (int64_t)batch * s.tr * s.tc >= (1LL << 31)) {
        delete L;
        return hdt_fail(HDT_ERR_SHAPE, "hdt_build_layout: batch * n_pos too large");
    }

    hipStream_t st = (hipStream_t)stream;
    const int B = batch, n = n_pos, tr = s.tr, tc = s.tc, wc = (tc + 31) / 32;
    hdt_status_t status = HDT_OK;
    (void)hipGetDevice(&L->device);
#define BUILD_TRY(expr)                                                                                 \
    do {                                                                                                \
        hipError_t _e = (expr);                                                                         \
        if (_e != hipSuccess) {                                                                         \
            status = hdt_fail(_e == hipErrorOutOfMemory ? HDT_ERR_OOM : HDT_ERR_HIP, "%s: %s", #expr, \
                              hipGetErrorString(_e));                                                   \
            goto fail;                                                                                  \
        }                                                                                               \
    } while (0)

    {
        Phase1 p = carve_phase1(nullptr, B, n, s.n_slots, tr, tc, wc);
        BUILD_TRY(pool_alloc(&L->arena, p.bytes, &L->arena_bytes));
        p = carve_phase1((char *)L->arena, B, n, s.n_slots, tr, tc, wc);

        // capacity of the per-tile arrays: exact for the dense baseline, else a guess
        int64_t cap = force_dense ? (int64_t)B * tr * tc : (int64_t)B * ((int64_t)tr * 8 + 64);
        {
            std::lock_guard<std::mutex> lk(g_pool_mutex);
            if (!force_dense && g_capacity_hint + g_capacity_hint / 8 > cap) cap = g_capacity_hint + g_capacity_hint / 8;
        }
        cap = cap > (int64_t)B * tr * tc ? (int64_t)B * tr * tc : cap;
        for (int attempt = 0; attempt < 2; attempt++) {
            if (cap >= (1LL << 31)) {
                status = hdt_fail(HDT_ERR_SHAPE, "hdt_build_layout: %lld candidate tiles", (long long)cap);
                goto fail;
            }
            Phase2 q = carve_phase2(nullptr, cap, bm, bn);
            BUILD_TRY(pool_alloc(&L->arena2, q.bytes, &L->arena2_bytes));
            q = carve_phase2((char *)L->arena2, cap, bm, bn);
            uint32_t ticket = 0;
            unsigned long long *report = report_slot(&ticket);
            if (!report) {
                status = hdt_fail(HDT_ERR_OOM, "hdt_build_layout: no pinned host memory for the build report");
                goto fail;
            }
            BUILD_TRY(hipMemsetAsync((char *)L->arena + p.zero_begin, 0, p.zero_end - p.zero_begin, st));
            {
                FrontArgs fa{d_level, d_parent, n, s.n_slots, bm, bn, tr, tc, wc, force_dense, no_sort, cap,
                             p.kperm, p.slot, p.cmin, p.cmax, p.cand, p.cand_ptr, q.c_row, q.q_cols, p.counters,
                             report, ticket};
                HdtTimer t("hdt_layout_front", st);
                hipLaunchKernelGGL(k_layout_front, dim3(B), dim3(kThreads), (size_t)kWaves * wc * sizeof(uint32_t), st,
                                   fa);
            }
            {
                const unsigned grid = (unsigned)(cap < 2048 ? (cap > 0 ? cap : 1) : 2048);
                HdtTimer t("hdt_layout_tile_bitmaps", st);
                hipLaunchKernelGGL(k_tile_bitmaps, dim3(grid), dim3(256), 0, st, d_level, d_parent, p.kperm, q.c_row,
                                   q.q_cols, p.counters, cap, n, s.n_slots, bm, bn, tr, q.bits, q.bits_rm, q.c_cnt,
                                   q.q_sub);
            }
            BUILD_TRY(hipGetLastError());
            // The host needs two facts before it can hand the layout out: whether the hierarchy was valid and
            // whether the per-tile arrays were large enough.  The front kernel knows both before it writes
            // the lists; it stores them into pinned host memory and the host polls that word instead of
            // draining the stream, so the bitmap kernel and whatever the caller enqueues next keep the GPU busy.
            unsigned long long word = 0;
            if (!wait_for_report(report, ticket, &word)) {
                // no word within the time limit: drain the stream and read the counters the slow way
                int32_t cnt[4] = {0, 0, 0, 0};
                BUILD_TRY(hipStreamSynchronize(st));
                BUILD_TRY(hipMemcpy(cnt, p.counters, sizeof(cnt), hipMemcpyDeviceToHost));
                word = report_word(ticket, cnt[CNT_ERR], (uint32_t)cnt[CNT_CAND]);
            }
            if ((word >> 39) & 1u) {
                BUILD_TRY(hipStreamSynchronize(st));  // the bitmap kernel still reads the arenas
                status = hdt_fail(HDT_ERR_HIERARCHY,
                                  "hdt_build_layout: level/parent arrays are not a valid hierarchy (level outside "
                                  "[-1, %d), parent outside [-1, n_pos), self-parent, pad with a parent, or pad parent)",
                                  HDT_MAX_LEVELS);
                goto fail;
            }
            const int64_t need = (int64_t)(word & 0xffffffffu);
            {
                std::lock_guard<std::mutex> lk(g_pool_mutex);
                if (!force_dense) g_capacity_hint = need;
            }
            if (need <= cap) {
                L->capacity = cap;
                L->n_entries = need;
                s.kperm = p.kperm;
                s.q_rowptr = p.cand_ptr;
                s.q_cols = q.q_cols;
                s.q_sub = q.q_sub;
                s.bits = q.bits;
                s.bits_rm = q.bits_rm;
                L->d_cnt = q.c_cnt;
                L->d_row = q.c_row;
                L->force_dense = force_dense;
                L->device_bytes = (int64_t)(L->arena_bytes + L->arena2_bytes);
                *out = L;
                return HDT_OK;
            }
            BUILD_TRY(hipStreamSynchronize(st));  // the bitmap kernel still writes the arrays about to be replaced
            // the guess was too small: once more with the exact size
            pool_free(L->arena2, L->arena2_bytes, L->device);
            L->arena2 = nullptr;
            cap = need;
        }
        status = hdt_fail(HDT_ERR_HIP, "hdt_build_layout: candidate count changed between two passes");
    }
fail:
    hdt_layout_release(L);
    L->magic = 0;
    delete L;
    return status;
#undef BUILD_TRY
}
