// hdt_build_layout: per-position level/parent ids -> block-sparse tile schedule, on the device.
//
// What is computed is fixed by the paper (Sec. 3.2: a position attends to parent, siblings and
// children; App. A.1, Alg. 1: sort keys by hierarchy level, partition into blocks, process a block
// only if its mask has a non-zero entry).  How it is computed is ours.  Two kinds of schedule:
//
//  key lists (the default): ONE kernel, key_lists, a workgroup per query tile.  It finds the keys the
//   tile's rows may attend to by scanning level[] / parent[] of the sample once, packs them in key order
//   (by level, ties in document order) into entries of tile_n keys, reserves the tile's slice of the
//   per-entry arrays with one atomic, and evaluates its entries exactly, by key columns (lane masks for
//   the MFMA kernels, pair count, 32x32 sub-block summary).  See the comment at the kernel.
//
//  windowed (Alg. 1 as printed: the key tiles are windows of the globally sorted key order; also the
//  dense baseline): four kernels.
//   sort_count / sort_scatter (one workgroup per 1024 positions)
//    1. key order: stable counting sort by level with wave ballots; the first kernel counts the levels
//       of every chunk, the second turns the counts into each chunk's first slot per level and hands
//       out the slots in document order;
//    2. per anchor, the range of sorted slots its children occupy (integer atomic min/max, one
//       pair of atomics per run of consecutive children);
//   candidates (one wave per query tile)
//    3. every allowed key of a row lies in one of <= 2 slot ranges (its siblings = the children of its
//       parent, and its own children) or is one of 2 single slots (itself, its parent), so a row marks
//       O(1) ranges in a bitmap over the key windows: the candidate windows of the query tile (exact for
//       documents laid out in pre-order, a superset for other forests); the workgroup reserves a slice
//       of the per-entry arrays with one atomic add and writes its candidates there;
//   tile_bitmaps (grid-stride over candidates)
//    4. every candidate is evaluated exactly, pair by pair (lane masks, pair count, sub-block summary,
//       the positions behind its key slots), so the result never depends on step 3 being tight.  A
//       candidate without any allowed pair keeps its list entry with an all-zero summary, which every
//       kernel skips; it is not counted as a tile and hdt_layout_export leaves it out.
//  The same two sort kernels produce the global key order of a key-list layout when hdt_layout_export
//  asks for it.
//
// The per-entry arrays are sized before the number of entries is known (a heuristic, raised by what
// earlier builds needed); the kernels check the capacity.  The kernel that reserves the entries reports
// the count (and whether the hierarchy was valid) through one word of pinned host memory as soon as it
// is known; the host waits for that word only, not for the stream, and repeats the build with the exact
// size in the rare case the guess was too small.
// Device memory comes from a small cache of earlier layouts' buffers.
#include <limits.h>
#include <stdio.h>
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
constexpr int kChunk = kThreads;              // positions per workgroup of the two sort kernels

// counters[CNT_ERR]: hierarchy error flag.  counters[CNT_CAND], counters[CNT_CAND + 1]: ONE 64-bit word,
// [39:0] list entries reserved so far, [63:40] workgroups that have reserved theirs: a single returning
// atomic gives a workgroup its slice and tells the last one that it is the last.
enum { CNT_ERR = 0, CNT_CAND = 2 };

// reserves `count` entries; returns the first one; *final_total >= 0 iff this was the last workgroup
__device__ __forceinline__ int reserve_entries(int32_t *counters, int count, int *final_total)
{
    unsigned long long *word = reinterpret_cast<unsigned long long *>(counters + CNT_CAND);
    const unsigned long long old = atomicAdd(word, (1ull << 40) + (unsigned long long)count);
    const int base = (int)(old & 0xffffffffffull);
    *final_total = (int)(old >> 40) == (int)gridDim.x - 1 ? base + count : -1;
    return base;
}

// What the candidate kernel reports to the host through pinned host memory: one 64-bit word
// [63:40] ticket of the build, [39] hierarchy error, [31:0] list entries needed.
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

__device__ __forceinline__ int bucket_of(int level) { return (level >= 0 && level < HDT_MAX_LEVELS) ? level : kBuckets - 1; }

// histogram of `bucket` over the lanes with `in`: lane k gets the number of lanes that hold bucket k
__device__ __forceinline__ int wave_bucket_count(bool in, int bucket)
{
    const int lane = threadIdx.x & 63;
    int mine = 0;
    unsigned long long remaining = __ballot(in);
    while (remaining) {
        const int leader = __ffsll((long long)remaining) - 1;
        const int bk = __builtin_amdgcn_readlane(bucket, leader);
        const unsigned long long m = __ballot(in && bucket == bk);
        if (lane == bk) mine = __popcll(m);
        remaining &= ~m;
    }
    return mine;
}

__device__ __forceinline__ void mark_tiles(uint32_t *bits, int tlo, int thi)
{
    for (int w = tlo >> 5; w <= (thi >> 5); w++) {
        const int lo = max(tlo, w << 5) & 31, hi = min(thi, (w << 5) + 31) & 31;
        const uint32_t m = (hi == 31 ? 0xffffffffu : ((1u << (hi + 1)) - 1u)) & ~((1u << lo) - 1u);
        atomicOr(&bits[w], m);
    }
}

struct SortArgs {
    const int32_t *level, *parent;
    int n, n_slots, nchunks, no_sort;
    int32_t *hist;  // [B][nchunks][kBuckets] positions of every level in every chunk of kChunk positions
    int32_t *kperm, *slot, *cmin, *cmax;
    int32_t *counters;
    int ranges;  // also compute the slot range of every node's children (windowed layouts)
    int32_t *level_copy;  // [B][n] or NULL: the layout's own copy of the level ids
};

// ---- sort, first half: validate, count the levels of each chunk ---------------------------------
__global__ __launch_bounds__(kThreads) void k_sort_count(SortArgs a)
{
    __shared__ int s_cnt[kWaves][kBuckets];
    const int b = blockIdx.x / a.nchunks, chunk = blockIdx.x - b * a.nchunks, n = a.n;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int i = chunk * kChunk + tid;
    const bool in = i < n;
    const size_t o = (size_t)b * n;
    int l = -1, p = -1;
    if (in) {
        l = a.level[o + i];
        p = a.parent[o + i];
        if (a.ranges) {
            a.cmin[o + i] = INT_MAX;
            a.cmax[o + i] = -1;
        }
        if (a.level_copy) a.level_copy[o + i] = l;
    }
    const bool bad = in && (l < -1 || l >= HDT_MAX_LEVELS || p < -1 || p >= n || p == i || (l < 0 && p != -1));
    if (__ballot(bad) && lane == 0) atomicOr(&a.counters[CNT_ERR], 1);
    if (chunk == a.nchunks - 1)
        for (int s = n + tid; s < a.n_slots; s += kThreads) a.kperm[(size_t)b * a.n_slots + s] = -1;
    const int mine = wave_bucket_count(in, bucket_of(l));
    if (lane < kBuckets) s_cnt[wave][lane] = mine;
    __syncthreads();
    if (tid < kBuckets) {
        int t = 0;
#pragma unroll
        for (int w = 0; w < kWaves; w++) t += s_cnt[w][tid];
        a.hist[((size_t)b * a.nchunks + chunk) * kBuckets + tid] = t;
    }
}

// ---- sort, second half: slots in document order; slot range of every node's children ------------
__global__ __launch_bounds__(kThreads) void k_sort_scatter(SortArgs a)
{
    __shared__ int s_cnt[kWaves][kBuckets], s_tot[kWaves][kBuckets], s_pre[kWaves][kBuckets];
    const int b = blockIdx.x / a.nchunks, chunk = blockIdx.x - b * a.nchunks, n = a.n;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int i = chunk * kChunk + tid;
    const bool in = i < n;
    const size_t o = (size_t)b * n;
    int l = -1, p = -1;
    if (in) {
        l = a.level[o + i];
        p = a.parent[o + i];
    }
    // what the parent check below needs, requested before the counting so that its latency hides there
    bool valid = in && l >= 0 && p >= 0 && p < n;
    const int lp = valid ? a.level[o + p] : 0;
    const int bucket = bucket_of(l);
    const int mine = wave_bucket_count(in, bucket);
    // lane k sums level k over the chunks this wave looks at: all of them, and those before this chunk
    int tot = 0, pre = 0;
    if (lane < kBuckets)
        for (int c = wave; c < a.nchunks; c += kWaves) {
            const int v = a.hist[((size_t)b * a.nchunks + c) * kBuckets + lane];
            tot += v;
            if (c < chunk) pre += v;
        }
    if (lane < kBuckets) {
        s_cnt[wave][lane] = mine;
        s_tot[wave][lane] = tot;
        s_pre[wave][lane] = pre;
    }
    __syncthreads();
    if (wave == 0) {  // first slot of every (level, wave of this chunk): level major, then chunk, then wave
        int t = 0, pr = 0;
        if (lane < kBuckets) {
#pragma unroll
            for (int w = 0; w < kWaves; w++) {
                t += s_tot[w][lane];
                pr += s_pre[w][lane];
            }
        }
        int incl = t;  // inclusive scan of the level totals over lanes
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int y = __shfl_up(incl, d);
            if (lane >= d) incl += y;
        }
        int run = incl - t + pr;
        if (lane < kBuckets) {
#pragma unroll
            for (int w = 0; w < kWaves; w++) {
                const int c = s_cnt[w][lane];
                s_cnt[w][lane] = run;
                run += c;
            }
        }
    }
    __syncthreads();
    const int mybase = lane < kBuckets ? s_cnt[wave][lane] : 0;
    int my_slot = i;
    {
        unsigned long long remaining = __ballot(in);
        while (remaining) {
            const int leader = __ffsll((long long)remaining) - 1;
            const int bk = __builtin_amdgcn_readlane(bucket, leader);
            const bool is_bk = in && bucket == bk;
            const unsigned long long m = __ballot(is_bk);
            const int first = __builtin_amdgcn_readlane(mybase, bk);
            if (is_bk) my_slot = first + __popcll(m & lanemask_lt());
            remaining &= ~m;
        }
    }
    if (a.no_sort) my_slot = i;
    if (in) {
        a.kperm[(size_t)b * a.n_slots + my_slot] = i;
    }
    if (!a.ranges) {
        if (valid && lp < 0) atomicOr(&a.counters[CNT_ERR], 1);  // a parent must be a real position
        return;
    }
    if (in) a.slot[o + i] = my_slot;
    // Slot range of every node's children.  Consecutive positions with the same parent and consecutive
    // slots (the tokens of a sentence, for one) form a run whose minimum and maximum are its first and
    // last slot: one atomic each per run.
    if (valid && lp < 0) {  // a parent must be a real position
        atomicOr(&a.counters[CNT_ERR], 1);
        valid = false;
    }
    const int sl = valid ? my_slot : -1;
    const int p_prev = __shfl_up(p, 1), s_prev = __shfl_up(sl, 1);
    const bool v_prev = __shfl_up((int)valid, 1) != 0;
    const bool head = lane == 0 || !v_prev || p_prev != p || s_prev + 1 != sl;
    const bool next_head = __shfl_down((int)(head || !valid), 1) != 0;  // lane+1 starts a new run (or is invalid)
    const bool tail = lane == 63 || next_head;
    if (valid && head) atomicMin(&a.cmin[o + p], sl);
    if (valid && tail) atomicMax(&a.cmax[o + p], sl);
}

struct CandArgs {
    const int32_t *level, *parent, *slot, *cmin, *cmax;
    int n, bm, bn, tr, tc, wc, force_dense, edges;
    int64_t capacity;
    int32_t *q_range;  // [B][tr][2]: first and one-past-last list entry of every query tile
    int32_t *c_row, *q_cols;
    int32_t *counters;
    unsigned long long *report;  // pinned host memory, written once by the last workgroup to get there
    uint32_t ticket;
};

// ---- candidate key tiles of every query tile: one wave per query tile, a bitmap per wave in LDS ----
__global__ __launch_bounds__(kThreads) void k_candidates(CandArgs a)
{
    extern __shared__ uint32_t s_bitmaps[];  // [kWaves][wc]
    __shared__ int s_n[kWaves];
    __shared__ int s_base;
    const int groups = (a.tr + kWaves - 1) / kWaves;
    const int b = blockIdx.x / groups, g = blockIdx.x - b * groups, n = a.n;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int bm = a.bm, bn = a.bn, tr = a.tr, tc = a.tc, wc = a.wc;
    const int I = g * kWaves + wave;
    const bool active = I < tr;
    const int32_t *level = a.level + (size_t)b * n, *parent = a.parent + (size_t)b * n;
    const int32_t *slot = a.slot + (size_t)b * n, *cmin = a.cmin + (size_t)b * n, *cmax = a.cmax + (size_t)b * n;
    uint32_t *wbits = s_bitmaps + (size_t)wave * wc;
    for (int w = lane; w < wc; w += 64) wbits[w] = 0;
    __builtin_amdgcn_wave_barrier();
    if (active && a.force_dense) {
        if (lane == 0) mark_tiles(wbits, 0, tc - 1);
    } else if (active) {
        // rows lane and lane + 64 of the tile; all loads of one dependency level are issued together
        int i2[2], sl2[2], p2[2], lo_c[2], hi_c[2];
        bool ok[2];
#pragma unroll
        for (int u = 0; u < 2; u++) {
            const int rr = lane + 64 * u;
            i2[u] = I * bm + rr;
            ok[u] = rr < bm && i2[u] < n;
            const int ii = ok[u] ? i2[u] : 0;
            ok[u] = ok[u] && level[ii] >= 0;
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
                if (a.edges & HDT_EDGE_UP) mark_tiles(wbits, sp2[u] / bn, sp2[u] / bn);  // its parent
                if ((a.edges & HDT_EDGE_SIBLING) && lo_s[u] <= hi_s[u] && lo_s[u] >= 0 && hi_s[u] < n)
                    mark_tiles(wbits, lo_s[u] / bn, hi_s[u] / bn);  // its siblings: the children of its parent
            }
            if ((a.edges & HDT_EDGE_DOWN) && lo_c[u] <= hi_c[u] && lo_c[u] >= 0 && hi_c[u] < n)
                mark_tiles(wbits, lo_c[u] / bn, hi_c[u] / bn);  // its children
        }
    }
    __builtin_amdgcn_wave_barrier();
    int cnt = 0;
    for (int w = lane; w < wc; w += 64) cnt += __popc(wbits[w]);
    cnt = wave_sum(cnt);
    if (lane == 0) s_n[wave] = cnt;
    __syncthreads();
    if (tid == 0) {
        int total = 0;
#pragma unroll
        for (int w = 0; w < kWaves; w++) total += s_n[w];
        // this workgroup's slice of the list arrays
        // this workgroup's slice of the list arrays; the last workgroup to get here knows the final count
        // and tells the host, which is waiting for exactly this word, while the lists and the bitmaps are
        // still being written (no device-scope fence: it would write back the whole L2 of this XCD)
        int final_total;
        s_base = reserve_entries(a.counters, total, &final_total);
        if (final_total >= 0) {
            const int err = __hip_atomic_load(&a.counters[CNT_ERR], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(a.report, report_word(a.ticket, err, (uint32_t)final_total), __ATOMIC_RELEASE,
                               __HIP_MEMORY_SCOPE_SYSTEM);
        }
    }
    __syncthreads();
    if (!active) return;
    int cbase = s_base;
    for (int w = 0; w < wave; w++) cbase += s_n[w];
    const size_t row = (size_t)b * tr + I;
    if (lane == 0) {
        a.q_range[2 * row] = cbase;
        a.q_range[2 * row + 1] = cbase + cnt;
    }
    int n_cand = 0;
    for (int w0 = 0; w0 < wc; w0 += 2) {
        const int w = w0 + (lane >> 5), bit = lane & 31;
        const uint32_t word = w < wc ? wbits[w] : 0u;
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

// ---- exact evaluation of one list entry pair by pair, by two waves (windowed layouts) ---------------
// Wave `wsub` (0 or 1) holds rows 64*wsub + lane of the query tile (position i, parent pi, rowok = a
// real position) and evaluates them against all keys (khalf < 0) or against one half of the entry's
// 32-key words (khalf = 0, 1); every wave holds the entry's keys, lane l the slots l and 64 + l (position
// and parent, -1 where the slot holds no key), which are broadcast by lane index while each lane tests
// its row against every key.  Outputs of entry c: per 32x32 sub-block the 16 x 64-bit lane masks the
// MFMA kernels apply to their accumulator registers (wave ballots), and through `part` (this wave's slot
// of a pair's scratch in LDS) the pair count and the sub-block summary, which the caller adds up after
// a barrier.
struct EntryPart {
    int cnt;
    uint32_t any, all;
    uint32_t col[4];  // entry_bitmaps only: key slots (32 per word) that some row of this wave may attend to
};

__device__ __forceinline__ uint32_t wave_or(uint32_t x)
{
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) x |= (uint32_t)__shfl_xor((int)x, d);
    return x;
}

__device__ __forceinline__ EntryPart entry_bitmaps(bool active, int64_t c, int wsub, int khalf, int lane, int i, int pi,
                                                   bool rowok,
                                                   const int (&kpos)[2], const int (&kpar)[2], int bm, int bn, int edges,
                                                   unsigned long long *bits_rm)
{
    const int wpr = bn >> 5, nrb = bm >> 5, nsub = nrb * wpr;
    // a disabled edge kind is a comparison against a value no key carries
    const int pi_sib = (edges & HDT_EDGE_SIBLING) && pi >= 0 ? pi : -3;  // my parent, for "same parent"
    const int pi_up = (edges & HDT_EDGE_UP) ? pi : -3;                   // my parent, for "is my parent"
    const int i_down = (edges & HDT_EDGE_DOWN) ? i : -3;                 // me, for "is my child"
    uint32_t w[4] = {0u, 0u, 0u, 0u};
    int cnt = 0;
#pragma unroll
    for (int wd = 0; wd < 4; wd++) {
        if (wd < wpr && (khalf < 0 || (wd * 2) / wpr == khalf)) {
            const int kp = kpos[wd >> 1], kq = kpar[wd >> 1];
            uint32_t out = 0;
#pragma unroll 8
            for (int cc = 0; cc < 32; cc++) {
                const int kj = __builtin_amdgcn_readlane(kp, (wd & 1) * 32 + cc);
                const int kr = __builtin_amdgcn_readlane(kq, (wd & 1) * 32 + cc);
                const bool ok = kj >= 0 && (kj == i || pi_sib == kr || pi_up == kj || kr == i_down);
                out |= (uint32_t)ok << cc;
            }
            w[wd] = rowok ? out : 0u;
            cnt += __popc(w[wd]);
        }
    }
    EntryPart part;
    part.cnt = wave_sum(cnt);
    part.any = part.all = 0;
#pragma unroll
    for (int wd = 0; wd < 4; wd++) part.col[wd] = wave_or(w[wd]);
    // register-major masks of sub-block (rblk, cblk), accumulator register e: bit l <=> row
    // rblk*32 + l%32, column cblk*32 + (l/32)*4 + 8*(e/4) + e%4
#pragma unroll
    for (int rr = 0; rr < 2; rr++) {
        const int rblk = 2 * wsub + rr;
        if (rblk < nrb) {
#pragma unroll
            for (int cblk = 0; cblk < 4; cblk++) {
                if (cblk < wpr && (khalf < 0 || (cblk * 2) / wpr == khalf)) {
                    const uint32_t x = (uint32_t)__shfl((int)w[cblk], rr * 32 + (lane & 31));
                    unsigned long long mine = 0;
#pragma unroll
                    for (int e = 0; e < 16; e++) {
                        const int bit = (lane >> 5) * 4 + 8 * (e >> 2) + (e & 3);
                        const unsigned long long m = __ballot((x >> bit) & 1u);
                        if (lane == e) mine = m;
                    }
                    const int sb = rblk * wpr + cblk;
                    if (active && lane < 16) bits_rm[((size_t)c * nsub + sb) * 16 + lane] = mine;
                    if (__ballot(x != 0u) != 0ull) part.any |= 1u << sb;
                    if (__ballot(x == 0xffffffffu) == ~0ull) part.all |= 1u << sb;
                }
            }
        }
    }
    return part;
}

// ---- bitmaps of a list entry by columns, one wave per 64 key slots ----------------------------------
// Lane c stands for key slot k0 + c and builds that key's COLUMN of the tile: bit r%32 of col[r/32] <=> row r
// may attend to it.  Rows see a key through their own parent in two ways - the key is that parent, or the
// key has the same parent - so for both the rows are R(v) = {rows whose parent is v}, with v the key's
// position or the key's parent; R is tabulated once per tile for the distinct parents of its rows (a
// handful, since the tokens of a sentence share theirs).  The key itself and the key's own parent are
// single rows.  The lane masks of the MFMA kernels need no transposition from there: mask e of sub-block
// (rblk, cblk) is the column word of key 32*cblk + 8*(e/4) + e%4 (lanes 0..31) next to that of key
// 32*cblk + 4 + 8*(e/4) + e%4 (lanes 32..63), so every lane stores its own words.
struct ParentTable {
    int n;
    const int *v;         // [n] distinct parents of the tile's rows
    const uint4 *rows;    // [n] the rows with that parent, 32 per word
};

__device__ __forceinline__ EntryPart entry_columns(int64_t c, int k0, int lane, const ParentTable &tab, const int *ek,
                                                   const int *ep, int row0, int bm, int bn, int edges,
                                                   unsigned long long *bits_rm)
{
    const int wpr = bn >> 5, nrb = bm >> 5, nsub = nrb * wpr;
    const int k = k0 + lane;
    const bool slot = k < bn;
    const int kj = slot ? ek[k] : -1, kr = slot ? ep[k] : -1;  // -1: no key
    const int v_up = (edges & HDT_EDGE_UP) ? kj : -1, v_sib = (edges & HDT_EDGE_SIBLING) ? kr : -1;
    uint32_t col[4] = {0u, 0u, 0u, 0u};
#pragma unroll 1
    for (int t = 0; t < tab.n; t++) {
        const int v = tab.v[t];  // >= 0
        const bool hit = v_up == v || v_sib == v;
        if (__ballot(hit) == 0ull) continue;
        const uint4 r = tab.rows[t];
        col[0] |= hit ? r.x : 0u;
        col[1] |= hit ? r.y : 0u;
        col[2] |= hit ? r.z : 0u;
        col[3] |= hit ? r.w : 0u;
    }
    // the key itself; the key's parent (the key is that row's child).  A key or a key's parent inside the
    // tile's range is a real position, hence a valid row.
    const int r_self = kj - row0, r_down = (edges & HDT_EDGE_DOWN) ? kr - row0 : -1;
    const bool has_self = kj >= 0 && r_self >= 0 && r_self < bm, has_down = kr >= 0 && r_down >= 0 && r_down < bm;
#pragma unroll
    for (int w = 0; w < 4; w++) {
        if (has_self && (r_self >> 5) == w) col[w] |= 1u << (r_self & 31);
        if (has_down && (r_down >> 5) == w) col[w] |= 1u << (r_down & 31);
    }
    EntryPart part;
    part.cnt = wave_sum(__popc(col[0]) + __popc(col[1]) + __popc(col[2]) + __popc(col[3]));
    part.any = part.all = 0;
    const int cblk = k >> 5, cc = k & 31, e = ((cc >> 3) << 2) | (cc & 3), hf = (cc >> 2) & 1;
    uint32_t *rm32 = reinterpret_cast<uint32_t *>(bits_rm + (size_t)c * nsub * 16);
#pragma unroll
    for (int rblk = 0; rblk < 4; rblk++) {
        if (rblk >= nrb) break;
        if (slot) rm32[((size_t)(rblk * wpr + cblk) * 16 + e) * 2 + hf] = col[rblk];
        const unsigned long long any = __ballot(col[rblk] != 0u), all = __ballot(col[rblk] == 0xffffffffu);
        const int sb = rblk * wpr + (k0 >> 5);  // lanes 0..31: sub-block sb, lanes 32..63: sb + 1
        if ((uint32_t)any) part.any |= 1u << sb;
        if ((uint32_t)(any >> 32)) part.any |= 2u << sb;
        if ((uint32_t)all == 0xffffffffu) part.all |= 1u << sb;
        if ((uint32_t)(all >> 32) == 0xffffffffu) part.all |= 2u << sb;
    }
    return part;
}

struct KeyListArgs {
    const int32_t *level, *parent;
    int n, bm, bn, tr, no_sort, edges;
    int64_t capacity;
    int32_t *q_range;  // [B][tr][2]
    int32_t *c_row, *q_keys, *q_kpar, *c_cnt;
    int32_t *level_copy, *parent_copy;  // the layout's own copy of the ids (the key order is sorted from it on demand)
    uint32_t *q_sub;
    unsigned long long *bits_rm;
    int32_t *counters;
    unsigned long long *report;      // pinned host memory
    unsigned long long *report_dev;  // the layout's own copy of the report
    uint32_t ticket;
    int self_reset;  // the counters are a slot that must be zero again when the build has reported
};

// Workgroup barrier for data exchanged through LDS only: unlike __syncthreads() it does not wait for this
// wave's global loads and stores (a store to HBM takes 2-3 us to be acknowledged).
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Sets the hierarchy error flag and waits for it to be set (a returning atomic): what this thread does next,
// a barrier in front of the workgroup's reservation, is then ordered behind it for the workgroup that reads
// the flag after the last reservation.
__device__ __forceinline__ void raise_error(int32_t *counters)
{
    const int old = atomicOr(&counters[CNT_ERR], 1);
    asm volatile("" ::"v"(old));
}

constexpr int kBatch = 8;
constexpr int kLdsKeys = 2048;  // key lists up to this length stay in LDS between the packing and the bitmaps

// ---- key lists: ONE kernel from level/parent to the finished entries, a workgroup per query tile ----
// Key j is needed by the tile iff it is one of the tile's rows, the parent of one (bitmap over the
// positions, in LDS), a child of one (its parent is a row of the tile) or a sibling of one (its parent
// is the parent of a row) - each kind only if its edges are enabled.  All four tests are exact, for any
// forest.  The workgroup scans level[] and
// parent[] of the whole sample once (two coalesced streams, nothing waits on a chain of dependent
// loads), keeps the needed positions as a bitmap, and packs them in KEY ORDER - by level, ties in
// document order, i.e. the order of kperm restricted to the needed keys - with a counting sort over the
// needed keys only: every wave counts the levels in its contiguous share, the counts are turned into
// first indices (level major, then wave), and after the workgroup has reserved its entries each wave
// hands out indices in document order.  The global key order is therefore not an input of this kernel.
// The workgroup then evaluates its own entries by key columns (entry_columns: lane masks, pair counts,
// summaries), one wave per 64 key slots.  It also validates its own rows.
// A list of up to kLdsKeys keys is packed into LDS while the reservation (a returning device-scope atomic,
// about 2 us) is in flight, copied to global memory from there, and evaluated from there; a longer list is
// packed straight into global memory once the reservation is back and read again from there.
// The workgroup has 1024 threads.  Tiles of up to 64 rows go to key_lists_pair below, two to a workgroup; where its
// bitmaps do not fit the LDS (documents beyond 64 K positions) they come here with 512 threads: they make twice
// the workgroups, and two of 512 threads share a compute unit where one of 1024 fills it (measured at 8192
// positions x 4 samples, 64-row tiles: 24 us against 28).
template <int kListThreads>
__global__ __launch_bounds__(kListThreads) void k_key_lists(KeyListArgs a)
{
    constexpr int kListWaves = kListThreads / 64;
    extern __shared__ uint32_t s_dyn[];  // [ceil(n/32)] parents of the tile's rows, then [2 * groups] needed positions
    __shared__ int2 s_row[128];          // (position, parent) of the tile's rows; position -2: no such row
    __shared__ int s_lcnt[kListWaves][kBuckets];  // needed keys per (wave, level), then their first index
    __shared__ int s_cnt[2][kListWaves];  // partial results of an entry's two waves (tile_n > 64), by parity of the round
    __shared__ uint32_t s_any[2][kListWaves], s_all[2][kListWaves];
    __shared__ int s_base, s_total, s_wtotal[kListWaves];
    __shared__ __attribute__((aligned(16))) int s_keys[kLdsKeys], s_kpar[kLdsKeys];
    __shared__ int s_tab_v[128], s_ntab;  // distinct parents of the tile's rows, and the rows of each
    __shared__ int s_first;               // first real row of the tile (a position), INT_MAX if it has none
    __shared__ uint4 s_tab_rows[128];
    const int b = blockIdx.x / a.tr, I = blockIdx.x - b * a.tr, n = a.n;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int bm = a.bm, bn = a.bn;
    const int32_t *level = a.level + (size_t)b * n, *parent = a.parent + (size_t)b * n;
    const int pw = (n + 31) >> 5, ng = (n + 63) >> 6;
    uint32_t *s_par = s_dyn, *s_need = s_dyn + pw;
    // kBatch groups of 64 positions at a time: all their loads are issued before the first is used, and those
    // of the first batch before anything else
    const int gpw = (ng + kListWaves - 1) / kListWaves;
    const int g0 = min(wave * gpw, ng), g1 = min(g0 + gpw, ng);
    int klv[kBatch], kp[kBatch];
    auto load_batch = [&](int gb) {
#pragma unroll
        for (int u = 0; u < kBatch; u++) {
            const int j = (gb + u) * 64 + lane;
            const bool ok = gb + u < g1 && j < n;
            klv[u] = ok ? level[j] : -1;
            kp[u] = ok ? parent[j] : -1;
        }
    };
    load_batch(g0);
    for (int w = tid; w < pw; w += kListThreads) s_par[w] = 0;
    if (tid == 0) s_first = INT_MAX;
    lds_barrier();
    const int row0 = I * bm;
    bool check_parent = false;
    int my_parent = 0;
    if (tid < 128) {
        int2 me = make_int2(-2, -2);
        if (tid < bm && row0 + tid < n) {
            const int i = row0 + tid;
            const int l = level[i], p = parent[i];
            a.level_copy[(size_t)b * n + i] = l;
            a.parent_copy[(size_t)b * n + i] = p;
            if (l < -1 || l >= HDT_MAX_LEVELS || p < -1 || p >= n || p == i || (l < 0 && p != -1))
                raise_error(a.counters);
            else if (l >= 0) {
                me = make_int2(i, p);
                atomicMin(&s_first, i);
                if (p >= 0) {
                    atomicOr(&s_par[p >> 5], 1u << (p & 31));
                    check_parent = true;
                    my_parent = p;
                }
            }
        }
        s_row[tid] = me;
    }
    const int parent_level = check_parent ? level[my_parent] : 0;  // looked at once the scan is under way
    lds_barrier();
    // A key is a real position, and so is the parent of one (or the build fails on the hierarchy): for both, being
    // a row of the tile is a matter of the range alone.  The two bitmap lookups are issued for every position,
    // needed or not, so that the loads of a whole batch are in flight together.
    auto in_tile = [&](int x) { return (unsigned)(x - row0) < (unsigned)bm; };
    const bool e_up = a.edges & HDT_EDGE_UP, e_sib = a.edges & HDT_EDGE_SIBLING, e_down = a.edges & HDT_EDGE_DOWN;
    int lcount = 0;  // lane k: needed keys of level k in this wave's share
    int wtotal = 0;  // needed keys in this wave's share
    for (int gb = g0; gb < g1; gb += kBatch) {
        if (gb != g0) load_batch(gb);
        bool need[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; u++) {  // groups past the share were loaded as pads
            const int j = (gb + u) * 64 + lane, pj = kp[u];
            const bool real = klv[u] >= 0 && j < n, has_parent = pj >= 0 && pj < n;
            const int jc = real ? j : 0, pc = has_parent ? pj : 0;
            const uint32_t wj = s_par[jc >> 5], wp = s_par[pc >> 5];
            const bool by_self = in_tile(j) | (e_up & (bool)((wj >> (jc & 31)) & 1u));
            const bool by_parent = has_parent & ((e_down & in_tile(pj)) | (e_sib & (bool)((wp >> (pc & 31)) & 1u)));
            need[u] = real & (by_self | by_parent);
        }
#pragma unroll
        for (int u = 0; u < kBatch; u++) {
            if (gb + u >= g1) break;
            const unsigned long long m = __ballot(need[u]);
            if (lane == 0) {
                s_need[2 * (gb + u)] = (uint32_t)m;
                s_need[2 * (gb + u) + 1] = (uint32_t)(m >> 32);
            }
            wtotal += __popcll(m);
            if (m != 0ull) lcount += wave_bucket_count(need[u], a.no_sort ? 0 : bucket_of(klv[u]));
        }
    }
    const bool one_batch = g1 - g0 <= kBatch;  // the registers still hold the wave's whole share
    if (lane < kBuckets) s_lcnt[wave][lane] = lcount;
    if (lane == 0) s_wtotal[wave] = wtotal;
    if (check_parent && parent_level < 0) raise_error(a.counters);  // a parent must be a real position
    lds_barrier();
    // This tile's slice of the per-entry arrays: reserved by wave 1 as soon as the length of the list is known,
    // used once the list has been packed.  The last workgroup to reserve knows the final count and tells the
    // host, which is waiting for exactly this word, while the lists and the bitmaps are still being written (no
    // device-scope fence: it would write back the whole L2 of this XCD).
    int reserved = 0, final_total = -1;
    if (wave == 1) {
        const int total = wave_sum(lane < kListWaves ? s_wtotal[lane] : 0);
        if (lane == 0) {
            s_total = total;
            reserved = reserve_entries(a.counters, (total + bn - 1) / bn, &final_total);
        }
    }
    if (wave == 2) {  // meanwhile: the table of the rows' parents (see entry_columns)
        const int2 ra = s_row[lane], rb = s_row[64 + lane];
        const int pa = ra.x >= 0 ? ra.y : -1, pb = rb.x >= 0 ? rb.y : -1;
        unsigned long long rem_a = __ballot(pa >= 0), rem_b = __ballot(pb >= 0);
        int nt = 0;
        while (rem_a | rem_b) {
            const int v = rem_a ? __builtin_amdgcn_readlane(pa, __ffsll((long long)rem_a) - 1)
                                : __builtin_amdgcn_readlane(pb, __ffsll((long long)rem_b) - 1);
            const unsigned long long ma = __ballot(pa == v), mb = __ballot(pb == v);
            if (lane == 0) {
                s_tab_v[nt] = v;
                s_tab_rows[nt] = make_uint4((uint32_t)ma, (uint32_t)(ma >> 32), (uint32_t)mb, (uint32_t)(mb >> 32));
            }
            rem_a &= ~ma;
            rem_b &= ~mb;
            nt++;
        }
        if (lane == 0) s_ntab = nt;
    }
    if (wave == 0) {  // first index of every (level, wave): level major, then wave
        int t = 0;
        if (lane < kBuckets) {
#pragma unroll
            for (int w = 0; w < kListWaves; w++) t += s_lcnt[w][lane];
        }
        int incl = t;  // inclusive scan of the level totals over lanes
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int y = __shfl_up(incl, d);
            if (lane >= d) incl += y;
        }
        int run = incl - t;
        if (lane < kBuckets) {
#pragma unroll
            for (int w = 0; w < kListWaves; w++) {
                const int c = s_lcnt[w][lane];
                s_lcnt[w][lane] = run;
                run += c;
            }
        }
    }
    lds_barrier();
    const int total = s_total, n_ent = (total + bn - 1) / bn;
    const bool in_lds = n_ent * bn <= kLdsKeys;
    // Slots behind the last key name no key: they hold ~f, f = the tile's first real row (a list with a key has
    // one), which is the row the attention kernels gather for such a slot.
    const int no_key = ~s_first;
    // hands out the indices of this wave's needed keys, in document order inside every level
    int mybase = lane < kBuckets ? s_lcnt[wave][lane] : 0;  // lane k: next index of level k in this wave
    auto pack = [&](bool to_lds, int32_t *keys, int32_t *kpars, int key_fit) {
        for (int gb = g0; gb < g1; gb += kBatch) {
            if (!one_batch) load_batch(gb);
#pragma unroll
            for (int u = 0; u < kBatch; u++) {
                if (gb + u >= g1) break;
                const int g = gb + u;
                const unsigned long long m = (unsigned long long)s_need[2 * g] | ((unsigned long long)s_need[2 * g + 1] << 32);
                if (m == 0ull) continue;
                const bool need = (m >> lane) & 1ull;
                const int bucket = a.no_sort ? 0 : bucket_of(klv[u]);
                int t = 0;
                unsigned long long remaining = m;
                while (remaining) {
                    const int leader = __ffsll((long long)remaining) - 1;
                    const int bk = __builtin_amdgcn_readlane(bucket, leader);
                    const bool is_bk = need && bucket == bk;
                    const unsigned long long mm = __ballot(is_bk);
                    const int first = __builtin_amdgcn_readlane(mybase, bk);
                    if (is_bk) t = first + __popcll(mm & lanemask_lt());
                    if (lane == bk) mybase += __popcll(mm);
                    remaining &= ~mm;
                }
                if (need) {
                    if (to_lds) {
                        s_keys[t] = g * 64 + lane;
                        s_kpar[t] = kp[u];
                    } else if (t < key_fit) {
                        keys[t] = g * 64 + lane;
                        kpars[t] = kp[u];
                    }
                }
            }
        }
    };
    if (in_lds) {  // while the reservation is in flight
        for (int t = total + tid; t < n_ent * bn; t += kListThreads) {  // tail of the last entry
            s_keys[t] = no_key;
            s_kpar[t] = -1;
        }
        pack(true, nullptr, nullptr, 0);
    }
    if (tid == 64) {
        s_base = reserved;
        if (final_total >= 0) {
            const int err = __hip_atomic_load(&a.counters[CNT_ERR], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (a.self_reset) {  // nobody touches the counters after the last reservation: clear them for the next build
                __hip_atomic_store(&a.counters[CNT_ERR], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(reinterpret_cast<unsigned long long *>(a.counters + CNT_CAND), 0ull, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            }
            const unsigned long long word = report_word(a.ticket, err, (uint32_t)final_total);
            *a.report_dev = word;
            __hip_atomic_store(a.report, word, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
        }
    }
    lds_barrier();
    const int64_t base = s_base;
    const size_t row = (size_t)b * a.tr + I;
    // entries past the capacity are not written, and the tile's range ends where they would begin: whoever walks
    // the lists stays inside the arrays (the host learns of the shortfall from the report and repeats the build
    // with larger arrays, or tells the caller of a deferred build to)
    const int64_t room = a.capacity - base;
    const int n_fit = room <= 0 ? 0 : (room < n_ent ? (int)room : n_ent);
    if (tid == 0) {
        const int32_t first = (int32_t)(room <= 0 ? a.capacity : base);
        a.q_range[2 * row] = first;
        a.q_range[2 * row + 1] = first + n_fit;
    }
    const int key_fit = n_fit * bn;
    for (int e = tid; e < n_fit; e += kListThreads) a.c_row[base + e] = (int32_t)row;
    int32_t *keys = a.q_keys + (size_t)base * bn, *kpars = a.q_kpar + (size_t)base * bn;
    if (in_lds) {
        for (int t = tid; t < key_fit; t += kListThreads) {
            keys[t] = s_keys[t];
            if (t < total) kpars[t] = s_kpar[t];
        }
    } else {
        for (int t = total + tid; t < key_fit; t += kListThreads) keys[t] = no_key;
        pack(false, keys, kpars, key_fit);
        // The keys were written to global memory by other waves of this workgroup; the barrier orders those
        // stores before the loads below at workgroup scope, which is all that is needed on one compute unit
        // (the loads also bypass the vector cache).
        __syncthreads();
    }
    // The entries of this tile out of LDS, one wave per 64 key slots; a list that did not fit is brought back
    // one round of entries at a time.
    const int wpe = (bn + 63) >> 6, per_round = kListWaves / wpe;  // waves per entry, entries per round
    const int quad = wave / wpe, k0 = (wave - quad * wpe) * 64;
    ParentTable tab;
    tab.n = s_ntab;
    tab.v = s_tab_v;
    tab.rows = s_tab_rows;
    int par = 0;
    for (int e0 = 0; e0 < n_fit; e0 += per_round, par ^= 1) {
        const int e = e0 + quad;
        int kb = e * bn;  // the entry's first key in s_keys, s_kpar
        if (!in_lds) {
            lds_barrier();  // the previous round's keys have been read
            for (int t = tid; t < per_round * bn; t += kListThreads) {
                const int gi = e0 * bn + t;
                int kk = -1, kq = -1;
                if (gi < key_fit) kk = __hip_atomic_load(&keys[gi], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (kk >= 0 && kk < n) kq = __hip_atomic_load(&kpars[gi], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                s_keys[t] = (kk >= 0 && kk < n) ? kk : -1;
                s_kpar[t] = kq;
            }
            lds_barrier();
            kb = quad * bn;
        }
        const bool active = e < n_fit;
        EntryPart part;
        part.cnt = 0;
        part.any = part.all = 0;
        if (active) part = entry_columns(base + e, k0, lane, tab, s_keys + kb, s_kpar + kb, row0, bm, bn, a.edges, a.bits_rm);
        if (wpe == 1) {
            if (active && lane == 0) {
                a.c_cnt[base + e] = part.cnt;
                a.q_sub[base + e] = part.any | (part.all << 16);
            }
            continue;
        }
        // two waves per entry: the slots of this parity were last read two rounds ago, in front of the previous
        // round's barrier
        if (lane == 0) {
            s_cnt[par][wave] = part.cnt;
            s_any[par][wave] = part.any;
            s_all[par][wave] = part.all;
        }
        lds_barrier();
        if (active && k0 == 0 && lane == 0) {
            a.c_cnt[base + e] = s_cnt[par][wave] + s_cnt[par][wave + 1];
            a.q_sub[base + e] = (s_any[par][wave] | s_any[par][wave + 1]) | ((s_all[par][wave] | s_all[par][wave + 1]) << 16);
        }
    }
}

// ---- key lists of TWO neighbouring query tiles of up to 64 rows per workgroup -------------------------
// Tiles of 64 rows make twice the query tiles, and every query tile's workgroup scans the ids of the whole
// sample; here the tiles 2P and 2P + 1 share one workgroup of 1024 threads and one scan, which tests every
// position against both tiles (two bitmaps of the rows' parents, two lists of needed keys); the two lists are
// then packed, reserved (one atomic for both: the entries of tile 2P, then those of tile 2P + 1) and evaluated
// as in key_lists, the waves working on the entries of both tiles side by side.  Same results, array by array
// (measured at 8192 positions x 4 samples, 64 x 32 tiles: 20 us against 24; 32768 positions: 43 against 48).
constexpr int kPairThreads = 1024, kPairWaves = kPairThreads / 64;

__global__ __launch_bounds__(kPairThreads) void k_key_lists_pair(KeyListArgs a)
{
    constexpr int W = kPairWaves;
    extern __shared__ uint32_t s_dyn[];  // 2 x [ceil(n/32)] parents of each tile's rows, then 2 x [2 * groups] needed positions
    __shared__ int2 s_row[128];          // (position, parent) of the rows: tile h at [64h, 64h + 64); position -2: no such row
    __shared__ int s_lcnt[2][W][kBuckets];
    __shared__ int s_cnt[2][W];
    __shared__ uint32_t s_any[2][W], s_all[2][W];
    __shared__ int s_base[2], s_total[2], s_wtotal[2][W];
    __shared__ __attribute__((aligned(16))) int s_keys[kLdsKeys], s_kpar[kLdsKeys];
    __shared__ int s_tab_v[2][64], s_ntab[2];
    __shared__ uint4 s_tab_rows[2][64];
    __shared__ int s_first[2];
    const int pairs = (a.tr + 1) >> 1;
    const int b = blockIdx.x / pairs, P = blockIdx.x - b * pairs, n = a.n;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int bm = a.bm, bn = a.bn;  // bm <= 64
    const int32_t *level = a.level + (size_t)b * n, *parent = a.parent + (size_t)b * n;
    const int pw = (n + 31) >> 5, ng = (n + 63) >> 6;
    uint32_t *s_par0 = s_dyn, *s_par1 = s_dyn + pw, *s_need0 = s_dyn + 2 * pw, *s_need1 = s_dyn + 2 * pw + 2 * ng;
    const int I0 = 2 * P, I1 = 2 * P + 1;
    const bool have1 = I1 < a.tr;  // the last pair of an odd number of tiles has one tile only
    const int row0_0 = I0 * bm, row0_1 = I1 * bm;
    const int bm1 = have1 ? bm : 0;
    const int gpw = (ng + W - 1) / W;
    const int g0 = min(wave * gpw, ng), g1 = min(g0 + gpw, ng);
    int klv[kBatch], kp[kBatch];
    auto load_batch = [&](int gb) {
#pragma unroll
        for (int u = 0; u < kBatch; u++) {
            const int j = (gb + u) * 64 + lane;
            const bool ok = gb + u < g1 && j < n;
            klv[u] = ok ? level[j] : -1;
            kp[u] = ok ? parent[j] : -1;
        }
    };
    load_batch(g0);
    for (int w = tid; w < 2 * pw; w += kPairThreads) s_dyn[w] = 0;
    if (tid < 2) s_first[tid] = INT_MAX;
    lds_barrier();
    bool check_parent = false;
    int my_parent = 0;
    if (tid < 128) {
        const int h = tid >> 6, r = tid & 63;
        const int i = (h ? row0_1 : row0_0) + r;
        int2 me = make_int2(-2, -2);
        if (r < (h ? bm1 : bm) && i < n) {
            const int l = level[i], p = parent[i];
            a.level_copy[(size_t)b * n + i] = l;
            a.parent_copy[(size_t)b * n + i] = p;
            if (l < -1 || l >= HDT_MAX_LEVELS || p < -1 || p >= n || p == i || (l < 0 && p != -1))
                raise_error(a.counters);
            else if (l >= 0) {
                me = make_int2(i, p);
                atomicMin(&s_first[h], i);
                if (p >= 0) {
                    atomicOr(&(h ? s_par1 : s_par0)[p >> 5], 1u << (p & 31));
                    check_parent = true;
                    my_parent = p;
                }
            }
        }
        s_row[tid] = me;
    }
    const int parent_level = check_parent ? level[my_parent] : 0;
    lds_barrier();
    const bool e_up = a.edges & HDT_EDGE_UP, e_sib = a.edges & HDT_EDGE_SIBLING, e_down = a.edges & HDT_EDGE_DOWN;
    int lcount0 = 0, lcount1 = 0, wtotal0 = 0, wtotal1 = 0;
    for (int gb = g0; gb < g1; gb += kBatch) {
        if (gb != g0) load_batch(gb);
        bool need0[kBatch], need1[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; u++) {
            const int j = (gb + u) * 64 + lane, pj = kp[u];
            const bool real = klv[u] >= 0 && j < n, has_parent = pj >= 0 && pj < n;
            const int jc = real ? j : 0, pc = has_parent ? pj : 0;
            const uint32_t wj0 = s_par0[jc >> 5], wp0 = s_par0[pc >> 5], wj1 = s_par1[jc >> 5], wp1 = s_par1[pc >> 5];
            const bool j_in0 = (unsigned)(j - row0_0) < (unsigned)bm, j_in1 = (unsigned)(j - row0_1) < (unsigned)bm1;
            const bool p_in0 = (unsigned)(pj - row0_0) < (unsigned)bm, p_in1 = (unsigned)(pj - row0_1) < (unsigned)bm1;
            const bool self0 = j_in0 | (e_up & (bool)((wj0 >> (jc & 31)) & 1u));
            const bool self1 = j_in1 | (e_up & (bool)((wj1 >> (jc & 31)) & 1u));
            const bool par0 = has_parent & ((e_down & p_in0) | (e_sib & (bool)((wp0 >> (pc & 31)) & 1u)));
            const bool par1 = has_parent & ((e_down & p_in1) | (e_sib & (bool)((wp1 >> (pc & 31)) & 1u)));
            need0[u] = real & (self0 | par0);
            need1[u] = real & (self1 | par1);
        }
#pragma unroll
        for (int u = 0; u < kBatch; u++) {
            if (gb + u >= g1) break;
            const unsigned long long m0 = __ballot(need0[u]), m1 = __ballot(need1[u]);
            if (lane == 0) {
                s_need0[2 * (gb + u)] = (uint32_t)m0;
                s_need0[2 * (gb + u) + 1] = (uint32_t)(m0 >> 32);
                s_need1[2 * (gb + u)] = (uint32_t)m1;
                s_need1[2 * (gb + u) + 1] = (uint32_t)(m1 >> 32);
            }
            wtotal0 += __popcll(m0);
            wtotal1 += __popcll(m1);
            const int bucket = a.no_sort ? 0 : bucket_of(klv[u]);
            if (m0 != 0ull) lcount0 += wave_bucket_count(need0[u], bucket);
            if (m1 != 0ull) lcount1 += wave_bucket_count(need1[u], bucket);
        }
    }
    const bool one_batch = g1 - g0 <= kBatch;
    if (lane < kBuckets) {
        s_lcnt[0][wave][lane] = lcount0;
        s_lcnt[1][wave][lane] = lcount1;
    }
    if (lane == 0) {
        s_wtotal[0][wave] = wtotal0;
        s_wtotal[1][wave] = wtotal1;
    }
    if (check_parent && parent_level < 0) raise_error(a.counters);
    lds_barrier();
    int reserved = 0, final_total = -1;
    if (wave == 1) {  // one reservation for both tiles
        const int t0 = wave_sum(lane < W ? s_wtotal[0][lane] : 0), t1 = wave_sum(lane < W ? s_wtotal[1][lane] : 0);
        if (lane == 0) {
            s_total[0] = t0;
            s_total[1] = t1;
            reserved = reserve_entries(a.counters, (t0 + bn - 1) / bn + (t1 + bn - 1) / bn, &final_total);
        }
    }
    if (wave == 2 || wave == 3) {  // the tables of the rows' parents, one per tile (64 rows each)
        const int h = wave - 2;
        const int2 ra = s_row[64 * h + lane];
        const int pa = ra.x >= 0 ? ra.y : -1;
        unsigned long long rem = __ballot(pa >= 0);
        int nt = 0;
        while (rem) {
            const int v = __builtin_amdgcn_readlane(pa, __ffsll((long long)rem) - 1);
            const unsigned long long ma = __ballot(pa == v);
            if (lane == 0) {
                s_tab_v[h][nt] = v;
                s_tab_rows[h][nt] = make_uint4((uint32_t)ma, (uint32_t)(ma >> 32), 0u, 0u);
            }
            rem &= ~ma;
            nt++;
        }
        if (lane == 0) s_ntab[h] = nt;
    }
    if (wave == 0 || wave == 4) {  // first index of every (level, wave) of a tile: level major, then wave
        const int h = wave >> 2;
        int t = 0;
        if (lane < kBuckets) {
#pragma unroll
            for (int w = 0; w < W; w++) t += s_lcnt[h][w][lane];
        }
        int incl = t;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int y = __shfl_up(incl, d);
            if (lane >= d) incl += y;
        }
        int run = incl - t;
        if (lane < kBuckets) {
#pragma unroll
            for (int w = 0; w < W; w++) {
                const int c = s_lcnt[h][w][lane];
                s_lcnt[h][w][lane] = run;
                run += c;
            }
        }
    }
    lds_barrier();
    const int total0 = s_total[0], total1 = s_total[1];
    const int n_ent0 = (total0 + bn - 1) / bn, n_ent1 = (total1 + bn - 1) / bn;
    const int koff1 = n_ent0 * bn;  // tile 1's list behind tile 0's in s_keys
    const bool in_lds = (n_ent0 + n_ent1) * bn <= kLdsKeys;
    const int no_key0 = ~s_first[0], no_key1 = ~s_first[1];
    // hands out the indices of this wave's needed keys of tile h, in document order inside every level
    auto pack = [&](int h, bool to_lds, int32_t *keys, int32_t *kpars, int key_fit) {
        int mybase = lane < kBuckets ? s_lcnt[h][wave][lane] : 0;
        const uint32_t *s_need = h ? s_need1 : s_need0;
        const int koff = h ? koff1 : 0;
        for (int gb = g0; gb < g1; gb += kBatch) {
            if (!one_batch) load_batch(gb);
#pragma unroll
            for (int u = 0; u < kBatch; u++) {
                if (gb + u >= g1) break;
                const int g = gb + u;
                const unsigned long long m = (unsigned long long)s_need[2 * g] | ((unsigned long long)s_need[2 * g + 1] << 32);
                if (m == 0ull) continue;
                const bool need = (m >> lane) & 1ull;
                const int bucket = a.no_sort ? 0 : bucket_of(klv[u]);
                int t = 0;
                unsigned long long remaining = m;
                while (remaining) {
                    const int leader = __ffsll((long long)remaining) - 1;
                    const int bk = __builtin_amdgcn_readlane(bucket, leader);
                    const bool is_bk = need && bucket == bk;
                    const unsigned long long mm = __ballot(is_bk);
                    const int first = __builtin_amdgcn_readlane(mybase, bk);
                    if (is_bk) t = first + __popcll(mm & lanemask_lt());
                    if (lane == bk) mybase += __popcll(mm);
                    remaining &= ~mm;
                }
                if (need) {
                    if (to_lds) {
                        s_keys[koff + t] = g * 64 + lane;
                        s_kpar[koff + t] = kp[u];
                    } else if (t < key_fit) {
                        keys[t] = g * 64 + lane;
                        kpars[t] = kp[u];
                    }
                }
            }
        }
    };
    if (in_lds) {  // while the reservation is in flight
        for (int t = total0 + tid; t < n_ent0 * bn; t += kPairThreads) {
            s_keys[t] = no_key0;
            s_kpar[t] = -1;
        }
        for (int t = total1 + tid; t < n_ent1 * bn; t += kPairThreads) {
            s_keys[koff1 + t] = no_key1;
            s_kpar[koff1 + t] = -1;
        }
        pack(0, true, nullptr, nullptr, 0);
        pack(1, true, nullptr, nullptr, 0);
    }
    if (tid == 64) {
        s_base[0] = reserved;
        s_base[1] = reserved + n_ent0;
        if (final_total >= 0) {
            const int err = __hip_atomic_load(&a.counters[CNT_ERR], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (a.self_reset) {
                __hip_atomic_store(&a.counters[CNT_ERR], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(reinterpret_cast<unsigned long long *>(a.counters + CNT_CAND), 0ull, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            }
            const unsigned long long word = report_word(a.ticket, err, (uint32_t)final_total);
            *a.report_dev = word;
            __hip_atomic_store(a.report, word, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
        }
    }
    lds_barrier();
    // per tile: its slice of the arrays, as far as it fits (see key_lists)
    int64_t base[2];
    int n_fit[2], key_fit[2];
    int32_t *keys[2], *kpars[2];
    for (int h = 0; h < 2; h++) {
        base[h] = s_base[h];
        const int n_ent = h ? n_ent1 : n_ent0;
        const int64_t room = a.capacity - base[h];
        n_fit[h] = room <= 0 ? 0 : (room < n_ent ? (int)room : n_ent);
        key_fit[h] = n_fit[h] * bn;
        keys[h] = a.q_keys + (size_t)(room <= 0 ? 0 : base[h]) * bn;
        kpars[h] = a.q_kpar + (size_t)(room <= 0 ? 0 : base[h]) * bn;
        const size_t row = (size_t)b * a.tr + (h ? I1 : I0);
        if (h == 1 && !have1) break;
        if (tid == 0) {
            const int32_t first = (int32_t)(room <= 0 ? a.capacity : base[h]);
            a.q_range[2 * row] = first;
            a.q_range[2 * row + 1] = first + n_fit[h];
        }
        for (int e = tid; e < n_fit[h]; e += kPairThreads) a.c_row[base[h] + e] = (int32_t)row;
    }
    if (!have1) n_fit[1] = key_fit[1] = 0;
    if (in_lds) {
        for (int t = tid; t < key_fit[0]; t += kPairThreads) {
            keys[0][t] = s_keys[t];
            if (t < total0) kpars[0][t] = s_kpar[t];
        }
        for (int t = tid; t < key_fit[1]; t += kPairThreads) {
            keys[1][t] = s_keys[koff1 + t];
            if (t < total1) kpars[1][t] = s_kpar[koff1 + t];
        }
    } else {
        for (int t = total0 + tid; t < key_fit[0]; t += kPairThreads) keys[0][t] = no_key0;
        for (int t = total1 + tid; t < key_fit[1]; t += kPairThreads) keys[1][t] = no_key1;
        pack(0, false, keys[0], kpars[0], key_fit[0]);
        pack(1, false, keys[1], kpars[1], key_fit[1]);
        __syncthreads();  // the keys were written by other waves of this workgroup (see key_lists)
    }
    // The entries of both tiles, one wave per 64 key slots.  Lists kept in LDS: the waves take the entries of both
    // tiles in one sequence; lists that did not fit are brought back tile by tile, a round of entries at a time.
    const int wpe = (bn + 63) >> 6, per_round = W / wpe;
    const int quad = wave / wpe, k0 = (wave - quad * wpe) * 64;
    ParentTable tab[2];
    for (int h = 0; h < 2; h++) {
        tab[h].n = s_ntab[h];
        tab[h].v = s_tab_v[h];
        tab[h].rows = s_tab_rows[h];
    }
    int par = 0;
    auto finish = [&](bool active, int64_t c, const EntryPart &part) {  // pair count and summary of entry c
        if (wpe == 1) {
            if (active && lane == 0) {
                a.c_cnt[c] = part.cnt;
                a.q_sub[c] = part.any | (part.all << 16);
            }
            return;
        }
        if (lane == 0) {
            s_cnt[par][wave] = part.cnt;
            s_any[par][wave] = part.any;
            s_all[par][wave] = part.all;
        }
        lds_barrier();
        if (active && k0 == 0 && lane == 0) {
            a.c_cnt[c] = s_cnt[par][wave] + s_cnt[par][wave + 1];
            a.q_sub[c] = (s_any[par][wave] | s_any[par][wave + 1]) | ((s_all[par][wave] | s_all[par][wave + 1]) << 16);
        }
        par ^= 1;
    };
    if (in_lds) {
        const int n_all = n_fit[0] + n_fit[1];
        for (int x0 = 0; x0 < n_all; x0 += per_round) {
            const int x = x0 + quad;
            const bool active = x < n_all;
            const int h = (active && x >= n_fit[0]) ? 1 : 0, e = x - (h ? n_fit[0] : 0);
            EntryPart part;
            part.cnt = 0;
            part.any = part.all = 0;
            if (active)
                part = entry_columns(base[h] + e, k0, lane, tab[h], s_keys + (h ? koff1 : 0) + e * bn,
                                     s_kpar + (h ? koff1 : 0) + e * bn, h ? row0_1 : row0_0, bm, bn, a.edges, a.bits_rm);
            finish(active, base[h] + e, part);
        }
    } else {
        for (int h = 0; h < 2; h++) {
            for (int e0 = 0; e0 < n_fit[h]; e0 += per_round) {
                const int e = e0 + quad;
                lds_barrier();  // the previous round's keys have been read
                for (int t = tid; t < per_round * bn; t += kPairThreads) {
                    const int gi = e0 * bn + t;
                    int kk = -1, kq = -1;
                    if (gi < key_fit[h]) kk = __hip_atomic_load(&keys[h][gi], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if (kk >= 0 && kk < n) kq = __hip_atomic_load(&kpars[h][gi], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    s_keys[t] = (kk >= 0 && kk < n) ? kk : -1;
                    s_kpar[t] = kq;
                }
                lds_barrier();
                const bool active = e < n_fit[h];
                EntryPart part;
                part.cnt = 0;
                part.any = part.all = 0;
                if (active)
                    part = entry_columns(base[h] + e, k0, lane, tab[h], s_keys + quad * bn, s_kpar + quad * bn, h ? row0_1 : row0_0,
                                         bm, bn, a.edges, a.bits_rm);
                finish(active, base[h] + e, part);
            }
        }
    }
}

// ---- bitmaps of a windowed layout: exact evaluation of every candidate tile -----------------------
// One candidate per workgroup iteration, a pair of waves (entry_bitmaps).  The keys of the tile are a
// window of the key order; the positions behind its slots are also written to q_keys, which is what the
// attention kernels read.
__global__ __launch_bounds__(128) void k_tile_bitmaps(const int32_t *__restrict__ level,
                                                      const int32_t *__restrict__ parent,
                                                      const int32_t *__restrict__ kperm,
                                                      const int32_t *__restrict__ c_row,
                                                      const int32_t *__restrict__ c_col, int32_t *q_keys,
                                                      const int32_t *__restrict__ counters, int64_t capacity,
                                                      int n, int n_slots, int bm, int bn, int tr, int edges,
                                                      int force_dense, unsigned long long *bits_rm, int32_t *c_cnt,
                                                      uint32_t *c_sub)
{
    __shared__ int s_cnt[2], s_first[2];
    __shared__ uint32_t s_any[2], s_all[2], s_col[2][4];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int64_t total = min((int64_t)(uint32_t)counters[CNT_CAND], capacity);  // low word of the combined counter
    for (int64_t c = blockIdx.x; c < total; c += gridDim.x) {
        const int row = c_row[c], J = c_col[c];
        const int b = row / tr, I = row - b * tr;
        const size_t o = (size_t)b * n;
        // keys: lane l holds slots l and 64 + l of the tile
        int kpos[2], kpar[2];
#pragma unroll
        for (int u = 0; u < 2; u++) {
            const int si = 64 * u + lane, s = J * bn + si;
            kpos[u] = (si < bn && s < n_slots) ? kperm[(size_t)b * n_slots + s] : -1;
        }
        // this lane's row
        const int r = wave * 64 + lane, i = I * bm + r;
        bool rowok = r < bm && i < n;
        const int ii = rowok ? i : 0;
        const int li = level[o + ii], pi = parent[o + ii];
        rowok = rowok && li >= 0;
#pragma unroll
        for (int u = 0; u < 2; u++) {
            const bool okp = kpos[u] >= 0 && kpos[u] < n;
            const int pp = okp ? kpos[u] : 0;
            const int lv = level[o + pp], pr = parent[o + pp];
            kpos[u] = (okp && lv >= 0) ? kpos[u] : -1;
            kpar[u] = (okp && lv >= 0) ? pr : -1;
        }
        const EntryPart part = entry_bitmaps(true, c, wave, -1, lane, i, pi, rowok, kpos, kpar, bm, bn, edges, bits_rm);
        const unsigned long long real_rows = __ballot(rowok);
        __syncthreads();  // the previous candidate's partial results have been read
        if (lane == 0) {
            s_cnt[wave] = part.cnt;
            s_any[wave] = part.any;
            s_all[wave] = part.all;
            s_first[wave] = real_rows ? I * bm + wave * 64 + __ffsll((long long)real_rows) - 1 : INT_MAX;
#pragma unroll
            for (int wd = 0; wd < 4; wd++) s_col[wave][wd] = part.col[wd];
        }
        __syncthreads();
        if (wave == 0) {
            // A slot keeps its key only if some row of the tile may attend to it; the others (pads, slots past the
            // key order, keys of no concern to this tile) hold ~f, f = the tile's first real row (0 if it has
            // none): the row the attention kernels gather in their place.
            const int f = s_first[0] != INT_MAX ? s_first[0] : (s_first[1] != INT_MAX ? s_first[1] : 0);
#pragma unroll
            for (int u = 0; u < 2; u++) {
                const int si = 64 * u + lane;
                const bool seen = ((s_col[0][si >> 5] | s_col[1][si >> 5]) >> (si & 31)) & 1u;
                if (si < bn) q_keys[(size_t)c * bn + si] = seen ? kpos[u] : ~f;
            }
        }
        if (tid == 0) {
            c_cnt[c] = s_cnt[0] + s_cnt[1];
            // the dense baseline computes every sub-block, allowed pairs or not
            const uint32_t any = force_dense ? (1u << ((bm >> 5) * (bn >> 5))) - 1u : (s_any[0] | s_any[1]);
            c_sub[c] = any | ((s_all[0] | s_all[1]) << 16);
        }
    }
}

// ---- device memory: a small cache of buffers of destroyed layouts ------------------------------
struct CachedBlock {
    void *ptr;
    size_t bytes;
    int device;
    HdtUsers users;  // work that may still read or write the block
};
std::mutex g_pool_mutex;
std::vector<CachedBlock> g_pool;
constexpr size_t kPoolMaxBlocks = 16;
constexpr size_t kPoolMaxBytes = (size_t)1 << 30;
int64_t g_capacity_hint = 0;  // candidates the last build needed

// Events for the fences: a free list, the events carry no timing.  The list and its mutex are never destroyed:
// fences held by the cache return their events when the process ends, in an order nobody controls.
std::mutex &g_event_mutex = *new std::mutex();
std::vector<hipEvent_t> &g_free_events = *new std::vector<hipEvent_t>();
hipStream_t g_last_build_stream = nullptr;  // where the most recent layout build was enqueued (under g_event_mutex)

hipError_t take_fence_event(hipEvent_t *ev)
{
    {
        std::lock_guard<std::mutex> lk(g_event_mutex);
        if (!g_free_events.empty()) {
            *ev = g_free_events.back();
            g_free_events.pop_back();
            return hipSuccess;
        }
    }
    return hipEventCreateWithFlags(ev, hipEventDisableTiming);
}

// Whatever is enqueued on `next` from here on runs after the work the users of a block had enqueued: the fences
// recorded at the release, and for the remembered streams an event recorded now (that covers more work than
// needed, never less); nothing at all for `next` itself (stream order), and no host wait.
hipError_t order_after(const HdtUsers &users, hipStream_t next)
{
    if (users.whole_device) return hipDeviceSynchronize();
    for (auto &f : users.fences) {
        if (f->stream == next) continue;
        const hipError_t e = hipStreamWaitEvent(next, f->ev, 0);
        if (e != hipSuccess) return e;
    }
    for (int i = 0; i < users.lazy.n; i++) {
        if (users.lazy.s[i] == next) continue;
        hipEvent_t ev;
        hipError_t e = take_fence_event(&ev);
        if (e != hipSuccess) return e;
        e = hipEventRecord(ev, users.lazy.s[i]);
        if (e == hipSuccess) e = hipStreamWaitEvent(next, ev, 0);
        {
            std::lock_guard<std::mutex> lk(g_event_mutex);
            g_free_events.push_back(ev);  // a later record on it does not disturb the wait already enqueued
        }
        if (e != hipSuccess) {  // e.g. the caller has destroyed that stream since: wait for everything instead
            (void)hipGetLastError();
            e = hipDeviceSynchronize();
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

hipError_t pool_alloc(void **out, size_t bytes, size_t *got, hipStream_t next_user)
{
    int dev = 0;
    (void)hipGetDevice(&dev);
    HdtUsers users;
    bool found = false;
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
            users = std::move(g_pool[best].users);
            g_pool.erase(g_pool.begin() + best);
            found = true;
        }
    }
    if (found) {
        const hipError_t e = order_after(users, next_user);
        if (e != hipSuccess) {  // the block goes back as it was
            std::lock_guard<std::mutex> lk(g_pool_mutex);
            g_pool.push_back({*out, *got, dev, std::move(users)});
            *out = nullptr;
        }
        return e;
    }
    *got = bytes;
    return hipMalloc(out, bytes);
}

void pool_free(void *ptr, size_t bytes, int device, const HdtUsers &users)
{
    if (!ptr) return;
    {
        std::lock_guard<std::mutex> lk(g_pool_mutex);
        size_t held = 0;
        for (auto &b : g_pool) held += b.bytes;
        if (g_pool.size() < kPoolMaxBlocks && held + bytes <= kPoolMaxBytes) {
            g_pool.push_back({ptr, bytes, device, users});
            return;
        }
    }
    (void)hipFree(ptr);  // waits for the device
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
    int32_t *kperm, *slot, *cmin, *cmax, *hist, *q_range, *counters, *level_copy, *parent_copy;
    unsigned long long *report_copy;
    size_t zero_begin, zero_end;  // byte range that must start at zero
    size_t bytes;
};

Phase1 carve_phase1(char *base, int B, int n, int n_slots, int tr, int nchunks)
{
    Carver c{base};
    Phase1 p;
    p.kperm = c.take<int32_t>((size_t)B * n_slots);
    p.slot = c.take<int32_t>((size_t)B * n);
    p.cmin = c.take<int32_t>((size_t)B * n);
    p.cmax = c.take<int32_t>((size_t)B * n);
    p.hist = c.take<int32_t>((size_t)B * nchunks * kBuckets);
    p.q_range = c.take<int32_t>((size_t)B * tr * 2);
    p.level_copy = c.take<int32_t>((size_t)B * n);
    p.parent_copy = c.take<int32_t>((size_t)B * n);
    p.report_copy = c.take<unsigned long long>(1);
    p.zero_begin = c.off;
    p.counters = c.take<int32_t>(64);
    p.zero_end = c.off;
    p.bytes = c.off;
    return p;
}

struct Phase2 {
    int32_t *q_cols, *c_row, *c_cnt, *q_keys, *q_kpar;
    uint32_t *q_sub;
    unsigned long long *bits_rm;
    size_t bytes;
};

Phase2 carve_phase2(char *base, int64_t cap, int bm, int bn)
{
    Carver c{base};
    Phase2 p;
    const size_t n = (size_t)cap, nsub = (size_t)(bm / 32) * (bn / 32);
    p.q_cols = c.take<int32_t>(n);
    p.q_sub = c.take<uint32_t>(n);
    p.c_row = c.take<int32_t>(n);
    p.c_cnt = c.take<int32_t>(n);
    p.q_keys = c.take<int32_t>(n * (size_t)bn);
    p.q_kpar = c.take<int32_t>(n * (size_t)bn);
    p.bits_rm = c.take<unsigned long long>(n * nsub * 16);
    p.bytes = c.off;
    return p;
}

// ---- the build's report from the device: words of pinned host memory, one per build in flight ----
constexpr int kReportSlots = 1024;
unsigned long long *g_reports = nullptr;  // never freed: a kernel may still write to it at exit
uint32_t g_ticket = 0;

unsigned long long *report_slot(uint32_t *ticket, uint32_t *ticket_before)
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
    unsigned long long *slot = g_reports + (size_t)(g_ticket % kReportSlots) * 8;  // one 64-byte line per slot
    *ticket_before = (uint32_t)(__atomic_load_n(slot, __ATOMIC_ACQUIRE) >> 40);
    if (*ticket_before == *ticket) {  // the ticket counter has wrapped around: a report of 2^24 builds ago
        __atomic_store_n(slot, 0ull, __ATOMIC_RELEASE);
        *ticket_before = 0;
    }
    return slot;
}

// The counters of a key-list build: device memory, one 256-byte slot per build in flight (chosen by the
// ticket, like the report word), zero whenever no build owns it: the kernel's last workgroup clears the slot
// before it reports, so a build needs no clearing launch of its own.  Never freed.
constexpr int kCounterDevices = 64;
int32_t *g_counter_slots[kCounterDevices] = {};

int32_t *counter_slot(int device, uint32_t ticket)
{
    if (device < 0 || device >= kCounterDevices) return nullptr;
    std::lock_guard<std::mutex> lk(g_pool_mutex);
    if (!g_counter_slots[device]) {
        void *ptr = nullptr;
        const size_t bytes = (size_t)kReportSlots * 64 * sizeof(int32_t);
        if (hipMalloc(&ptr, bytes) != hipSuccess || hipMemset(ptr, 0, bytes) != hipSuccess) {
            (void)hipGetLastError();
            if (ptr) (void)hipFree(ptr);
            return nullptr;
        }
        g_counter_slots[device] = static_cast<int32_t *>(ptr);
    }
    return g_counter_slots[device] + (size_t)(ticket % kReportSlots) * 64;
}

// polls the word until it carries this build's ticket; false after 10 s without it, or at once when the slot
// has been taken over by a later build (it then holds neither this ticket nor the one it held before)
bool wait_for_report(const unsigned long long *slot, uint32_t ticket, uint32_t ticket_before, unsigned long long *word)
{
    const auto t0 = std::chrono::steady_clock::now();
    for (uint64_t spins = 0;; spins++) {
        const unsigned long long w = __atomic_load_n(slot, __ATOMIC_ACQUIRE);
        if ((uint32_t)(w >> 40) == ticket) {
            *word = w;
            return true;
        }
        if ((uint32_t)(w >> 40) != ticket_before) return false;
        if ((spins & 0x3ff) == 0x3ff && std::chrono::steady_clock::now() - t0 > std::chrono::seconds(10)) return false;
        __builtin_ia32_pause();
    }
}

const char kHierarchyText[] =
    "level/parent arrays are not a valid hierarchy (level outside [-1, 32), parent outside [-1, n_pos), self-parent, "
    "pad with a parent, or pad parent)";

}  // namespace

// What a deferred build's report says, read at most once per layout.
static hdt_status_t resolve_one(const hdt_layout_t *L, bool wait)
{
    static std::mutex resolve_mutex;
    std::lock_guard<std::mutex> lk(resolve_mutex);
    if (L->pending) {
        unsigned long long word = __atomic_load_n(L->report, __ATOMIC_ACQUIRE);
        bool have = (uint32_t)(word >> 40) == L->ticket;
        if (!have && !wait) return HDT_OK;
        if (!have) have = wait_for_report(L->report, L->ticket, L->ticket_before, &word);
        if (!have) {
            // the slot has gone to a later build (or nothing came for 10 s): the copy in the layout's own memory
            int dev = 0;
            HDT_HIP_TRY(hipGetDevice(&dev));
            if (dev != L->device) HDT_HIP_TRY(hipSetDevice(L->device));
            hipError_t e = hipDeviceSynchronize();
            if (e == hipSuccess) e = hipMemcpy(&word, L->report_dev, sizeof(word), hipMemcpyDeviceToHost);
            if (dev != L->device) (void)hipSetDevice(dev);
            if (e != hipSuccess) return hdt_fail(HDT_ERR_HIP, "hdt_layout_resolve: %s", hipGetErrorString(e));
            if ((uint32_t)(word >> 40) != L->ticket)
                return hdt_fail(HDT_ERR_HIP, "hdt_layout_resolve: the build kernel finished without its report");
        }
        const int64_t need = (int64_t)(word & 0xffffffffu);
        L->entries_needed = need;
        if ((word >> 39) & 1u) {
            L->build_status = HDT_ERR_HIERARCHY;
            snprintf(L->build_error, sizeof(L->build_error), "deferred hdt_build_layout: %s", kHierarchyText);
        } else if (need > L->capacity) {
            L->build_status = HDT_ERR_SHAPE;
            snprintf(L->build_error, sizeof(L->build_error),
                     "deferred hdt_build_layout: the schedule needs %lld list entries, the layout holds %lld "
                     "(build again with opts->capacity)", (long long)need, (long long)L->capacity);
        } else {
            L->n_entries = need;
        }
        if (!((word >> 39) & 1u)) {
            std::lock_guard<std::mutex> lk2(g_pool_mutex);
            g_capacity_hint = need;
        }
        L->pending = false;
    }
    if (L->build_status != HDT_OK) return hdt_fail(L->build_status, "%s", L->build_error);
    return HDT_OK;
}

hdt_status_t hdt_layout_resolve(const hdt_layout_t *L, bool wait)
{
    if (hdt_status_t st = resolve_one(L, wait)) return st;
    if (L->transposed) return resolve_one(L->transposed, wait);
    return HDT_OK;
}

hipError_t hdt_pool_alloc(void **out, size_t bytes, size_t *got, hipStream_t next_user)
{
    return pool_alloc(out, bytes, got, next_user);
}

void hdt_layout_release(hdt_layout_t *L, const HdtUsers &users)
{
    pool_free(L->arena, L->arena_bytes, L->device, users);
    pool_free(L->arena2, L->arena2_bytes, L->device, users);
    L->arena = L->arena2 = nullptr;
}

HdtFence::~HdtFence()
{
    std::lock_guard<std::mutex> lk(g_event_mutex);
    g_free_events.push_back(ev);
}

HdtUsers hdt_users_at_release(const HdtStreams &streams)
{
    HdtUsers u;
    if (streams.more) {
        u.whole_device = true;
        return u;
    }
    hipStream_t builds;
    {
        std::lock_guard<std::mutex> lk(g_event_mutex);
        builds = g_last_build_stream;
    }
    for (int i = 0; i < streams.n; i++) {
        if (streams.s[i] == builds) {
            u.lazy.add(streams.s[i]);
            continue;
        }
        hipEvent_t ev;
        if (take_fence_event(&ev) != hipSuccess || hipEventRecord(ev, streams.s[i]) != hipSuccess) {
            (void)hipGetLastError();
            u.whole_device = true;  // the next owner waits for the device instead
            return u;
        }
        u.fences.push_back(std::shared_ptr<HdtFence>(new HdtFence{ev, streams.s[i]}));
    }
    return u;
}

// a buffer that only a build on `st` has touched
static HdtUsers only_stream(hipStream_t st)
{
    HdtUsers u;
    u.lazy.add(st);
    return u;
}

void hdt_note_build_stream(hipStream_t st)
{
    std::lock_guard<std::mutex> lk(g_event_mutex);
    g_last_build_stream = st;
}

static std::mutex g_streams_mutex;  // attention calls on one layout may come from several host threads

void hdt_layout_note_stream(const hdt_layout_t *L, hipStream_t st)
{
    std::lock_guard<std::mutex> lk(g_streams_mutex);
    L->streams.add(st);
}

HdtStreams hdt_layout_streams(const hdt_layout_t *L)
{
    std::lock_guard<std::mutex> lk(g_streams_mutex);
    return L->streams;
}

// Surviving tiles and allowed pairs per sample, summed on the host from the query tile and the pair
// count of every list entry (two adjacent device arrays): cheaper than thousands of device atomics on
// a handful of addresses, and only paid by callers that ask.
hdt_status_t hdt_layout_stats(const hdt_layout_t *L)
{
    static std::mutex stats_mutex;
    std::lock_guard<std::mutex> lk(stats_mutex);
    if (L->stats_ready) return HDT_OK;
    if (hdt_status_t st = hdt_layout_resolve(L, true)) return st;
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

// The key order of a layout built from key lists: sorted from the layout's own copy of the ids by the
// first caller that asks for it (the build itself never needs it).  Waits for the device.
hdt_status_t hdt_layout_ensure_kperm(const hdt_layout_t *L)
{
    static std::mutex kperm_mutex;
    std::lock_guard<std::mutex> lk(kperm_mutex);
    if (L->kperm_ready || L->s.batch == 0 || L->s.n_pos == 0) return HDT_OK;
    int dev = 0;
    HDT_HIP_TRY(hipGetDevice(&dev));
    if (dev != L->device) HDT_HIP_TRY(hipSetDevice(L->device));
    hipError_t e = hipDeviceSynchronize();
    if (e == hipSuccess) {
        const int B = L->s.batch, n = L->s.n_pos, nchunks = (n + kChunk - 1) / kChunk;
        SortArgs sa{L->level_copy, L->parent_copy, n, L->s.n_slots, nchunks, L->no_sort, L->sort_hist,
                    const_cast<int32_t *>(L->s.kperm), nullptr, nullptr, nullptr, L->sort_counters, 0, nullptr};
        hipLaunchKernelGGL(k_sort_count, dim3((unsigned)B * nchunks), dim3(kThreads), 0, nullptr, sa);
        hipLaunchKernelGGL(k_sort_scatter, dim3((unsigned)B * nchunks), dim3(kThreads), 0, nullptr, sa);
        e = hipGetLastError();
        if (e == hipSuccess) e = hipDeviceSynchronize();
    }
    if (dev != L->device) (void)hipSetDevice(dev);
    if (e != hipSuccess) return hdt_fail(HDT_ERR_HIP, "hdt_layout_ensure_kperm: %s", hipGetErrorString(e));
    L->kperm_ready = true;
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

static hdt_status_t build_one(const int32_t *d_level, const int32_t *d_parent, int32_t batch, int32_t n_pos,
                              const hdt_layout_opts_t *opts, int edges, void *stream, hdt_layout_t **out);

static int swap_up_down(int edges)
{
    return (edges & HDT_EDGE_SIBLING) | ((edges & HDT_EDGE_UP) ? HDT_EDGE_DOWN : 0) | ((edges & HDT_EDGE_DOWN) ? HDT_EDGE_UP : 0);
}

extern "C" __attribute__((visibility("default"))) hdt_status_t hdt_build_layout(const int32_t *d_level,
                                                                                 const int32_t *d_parent,
                                                                                 int32_t batch, int32_t n_pos,
                                                                                 const hdt_layout_opts_t *opts,
                                                                                 void *stream, hdt_layout_t **out)
{
    if (!out) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_build_layout: out is NULL");
    *out = nullptr;
    int edges = opts && opts->edges ? opts->edges : HDT_EDGE_ALL;
    if (edges & ~HDT_EDGE_ALL) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_build_layout: edges = %d", edges);
    hdt_layout_t *L = nullptr;
    hdt_status_t st = build_one(d_level, d_parent, batch, n_pos, opts, edges, stream, &L);
    if (st != HDT_OK) return st;
    if (swap_up_down(edges) != edges) {
        // a directed mask: the backward pass also needs the schedule of its transpose, which is the same
        // construction with the parent and child kinds exchanged
        st = build_one(d_level, d_parent, batch, n_pos, opts, swap_up_down(edges), stream, &L->transposed);
        if (st != HDT_OK) {
            (void)hdt_layout_destroy(L);
            return st;
        }
        L->device_bytes += L->transposed->device_bytes;
    }
    *out = L;
    return HDT_OK;
}

static hdt_status_t build_one(const int32_t *d_level, const int32_t *d_parent, int32_t batch, int32_t n_pos,
                              const hdt_layout_opts_t *opts, int edges, void *stream, hdt_layout_t **out)
{
    *out = nullptr;
    if (batch < 0 || n_pos < 0) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_build_layout: negative size");
    if (n_pos > (1 << 19)) return hdt_fail(HDT_ERR_SHAPE, "hdt_build_layout: n_pos %d > 2^19", n_pos);
    int bm = 128, bn = 64, force_dense = 0, no_sort = 0, windowed = 0;
    bool deferred = false;
    int64_t capacity_opt = 0;
    if (opts) {
        if (opts->tile_m) bm = opts->tile_m;
        if (opts->tile_n) bn = opts->tile_n;
        force_dense = opts->force_dense != 0;
        no_sort = opts->no_sort != 0;
        windowed = opts->windowed != 0 || force_dense;
        if (opts->capacity < 0) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_build_layout: capacity = %lld", (long long)opts->capacity);
        capacity_opt = opts->capacity;
        deferred = opts->deferred != 0 && !windowed;  // the windowed kernels are launched from what the first reports
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
    L->kperm_ready = true;
    L->no_sort = 0;
    L->sort_hist = L->sort_counters = nullptr;
    L->level_copy = L->parent_copy = nullptr;
    L->force_dense = force_dense;
    L->windowed = windowed;
    L->edges = edges;
    L->cross = 0;
    L->cross_level_mask = 0;
    L->transposed = nullptr;
    L->compact = nullptr;
    L->cross_sel = L->cross_count = L->cross_rank = nullptr;
    L->n_compact = 0;
    L->device_bytes = 0;
    L->device = 0;
    L->pending = false;
    L->build_status = HDT_OK;
    L->entries_needed = 0;
    L->build_error[0] = 0;
    L->report = L->report_dev = nullptr;
    L->ticket = L->ticket_before = 0;
    HdtSchedule &s = L->s;
    memset(&s, 0, sizeof(s));
    s.batch = batch;
    s.n_pos = n_pos;
    s.n_kv = n_pos;
    s.bm = bm;
    s.bn = bn;
    s.wpr = bn / 32;
    s.tr = empty ? 0 : (n_pos + bm - 1) / bm;
    s.tc = empty ? 0 : (n_pos + bn - 1) / bn;
    s.n_slots = s.tc * bn;
    s.n_own = n_pos;
    s.tr_own = s.tr;
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
    L->streams.add(st);
    hdt_note_build_stream(st);
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
        const int nchunks = (n + kChunk - 1) / kChunk, groups = (tr + kWaves - 1) / kWaves;
        Phase1 p = carve_phase1(nullptr, B, n, s.n_slots, tr, nchunks);
        BUILD_TRY(pool_alloc(&L->arena, p.bytes, &L->arena_bytes, st));
        p = carve_phase1((char *)L->arena, B, n, s.n_slots, tr, nchunks);

        // The schedule as far as the host knows it before the device has reported.
        auto adopt = [&](const Phase2 &q, int64_t cap) {
            L->capacity = cap;
            s.kperm = p.kperm;
            L->kperm_ready = windowed != 0;
            L->no_sort = no_sort;
            L->sort_hist = p.hist;
            L->sort_counters = p.counters;
            L->level_copy = p.level_copy;
            L->parent_copy = p.parent_copy;
            s.q_range = p.q_range;
            s.q_cols = q.q_cols;
            s.q_keys = q.q_keys;
            s.q_sub = q.q_sub;
            s.bits_rm = q.bits_rm;
            s.row_flag = p.level_copy;
            L->d_cnt = q.c_cnt;
            L->d_row = q.c_row;
            L->force_dense = force_dense;
            L->device_bytes = (int64_t)(L->arena_bytes + L->arena2_bytes);
        };
        // capacity of the per-tile arrays: exact for the dense baseline, the caller's if given, else a guess raised
        // by what earlier builds needed.  A deferred build cannot be repeated by this call, so it takes what no
        // document can exceed (every query tile listing every key) as far as that stays below 256 MiB.
        const int64_t cap_bound = (int64_t)B * tr * tc;
        int64_t cap = force_dense ? cap_bound : (int64_t)B * ((int64_t)tr * 8 + 64);
        if (!force_dense) {
            std::lock_guard<std::mutex> lk(g_pool_mutex);
            if (g_capacity_hint + g_capacity_hint / 8 > cap) cap = g_capacity_hint + g_capacity_hint / 8;
        }
        if (deferred) {
            const int64_t per_entry = (int64_t)carve_phase2(nullptr, 1024, bm, bn).bytes / 1024 + 1;
            cap = std::max(cap, ((int64_t)256 << 20) / per_entry);
        }
        if (!force_dense && capacity_opt > 0) cap = capacity_opt;
        cap = cap > cap_bound ? cap_bound : cap;
        for (int attempt = 0; attempt < 2; attempt++) {
            if (cap >= (1LL << 31)) {
                status = hdt_fail(HDT_ERR_SHAPE, "hdt_build_layout: %lld candidate tiles", (long long)cap);
                goto fail;
            }
            Phase2 q = carve_phase2(nullptr, cap, bm, bn);
            BUILD_TRY(pool_alloc(&L->arena2, q.bytes, &L->arena2_bytes, st));
            q = carve_phase2((char *)L->arena2, cap, bm, bn);
            uint32_t ticket = 0, ticket_before = 0;
            unsigned long long *report = report_slot(&ticket, &ticket_before);
            if (!report) {
                status = hdt_fail(HDT_ERR_OOM, "hdt_build_layout: no pinned host memory for the build report");
                goto fail;
            }
            // the windowed kernels count in the arena, cleared here; a key-list build counts in a slot that is
            // already clear (if there is none, in the arena as well)
            int32_t *slot_counters = windowed ? nullptr : counter_slot(L->device, ticket);
            if (!slot_counters)
                BUILD_TRY(hipMemsetAsync((char *)L->arena + p.zero_begin, 0, p.zero_end - p.zero_begin, st));
            if (windowed) {
                SortArgs sa{d_level, d_parent, n, s.n_slots, nchunks, no_sort, p.hist, p.kperm, p.slot, p.cmin,
                            p.cmax, p.counters, 1, p.level_copy};
                {
                    HdtTimer t("hdt_layout_sort_count", st);
                    hipLaunchKernelGGL(k_sort_count, dim3((unsigned)B * nchunks), dim3(kThreads), 0, st, sa);
                }
                {
                    HdtTimer t("hdt_layout_sort_scatter", st);
                    hipLaunchKernelGGL(k_sort_scatter, dim3((unsigned)B * nchunks), dim3(kThreads), 0, st, sa);
                }
                CandArgs ca{d_level, d_parent, p.slot, p.cmin, p.cmax, n, bm, bn, tr, tc, wc, force_dense, edges, cap,
                            p.q_range, q.c_row, q.q_cols, p.counters, report, ticket};
                HdtTimer t("hdt_layout_candidates", st);
                hipLaunchKernelGGL(k_candidates, dim3((unsigned)B * groups), dim3(kThreads),
                                   (size_t)kWaves * wc * sizeof(uint32_t), st, ca);
            } else {
                // one kernel from the ids to the finished entries; the global key order is not needed for it
                // and is sorted from the layout's copy of the ids only when someone asks (hdt_layout_export)
                KeyListArgs ka{d_level, d_parent, n, bm, bn, tr, no_sort, edges, cap, p.q_range, q.c_row, q.q_keys, q.q_kpar,
                               q.c_cnt, p.level_copy, p.parent_copy, q.q_sub, q.bits_rm,
                               slot_counters ? slot_counters : p.counters, report, p.report_copy, ticket,
                               slot_counters != nullptr};
                const size_t lds = ((size_t)(n + 31) / 32 + (size_t)2 * ((n + 63) / 64)) * sizeof(uint32_t);
                const bool small_wg = bm <= 64;
                // tiles of up to 64 rows: two per workgroup, as long as the two sets of bitmaps fit the LDS beside the
                // kernel's static arrays (documents of up to 64 K positions)
                const bool pair = small_wg && 2 * lds <= 32 * 1024;
                if (!pair && lds > 32 * 1024)  // with the kernel's static arrays: beyond the 64 KB a launch gets by default
                    BUILD_TRY(hipFuncSetAttribute(small_wg ? (const void *)k_key_lists<512> : (const void *)k_key_lists<1024>,
                                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
                HdtTimer t("hdt_layout_key_lists", st);
                if (pair)
                    hipLaunchKernelGGL(k_key_lists_pair, dim3((unsigned)B * ((tr + 1) / 2)), dim3(kPairThreads), 2 * lds, st, ka);
                else if (small_wg)
                    hipLaunchKernelGGL(k_key_lists<512>, dim3((unsigned)B * tr), dim3(512), lds, st, ka);
                else
                    hipLaunchKernelGGL(k_key_lists<1024>, dim3((unsigned)B * tr), dim3(1024), lds, st, ka);
            }
            if (windowed) {
                const unsigned grid = (unsigned)(cap < 2048 ? (cap > 0 ? cap : 1) : 2048);
                HdtTimer t("hdt_layout_tile_bitmaps", st);
                hipLaunchKernelGGL(k_tile_bitmaps, dim3(grid), dim3(128), 0, st, d_level, d_parent, p.kperm, q.c_row,
                                   q.q_cols, q.q_keys, p.counters, cap, n, s.n_slots, bm, bn, tr, edges, force_dense,
                                   q.bits_rm, q.c_cnt, q.q_sub);
            }
            BUILD_TRY(hipGetLastError());
            if (deferred) {
                // The layout goes out as it is.  What the device reports (through the same word of pinned host
                // memory, and a copy in the layout's own memory) is read by hdt_layout_resolve, when someone asks.
                adopt(q, cap);
                L->n_entries = 0;
                L->entries_needed = -1;
                L->pending = true;
                L->report = report;
                L->report_dev = p.report_copy;
                L->ticket = ticket;
                L->ticket_before = ticket_before;
                *out = L;
                return HDT_OK;
            }
            // The host needs two facts before it can hand the layout out: whether the hierarchy was valid and
            // whether the per-tile arrays were large enough.  The candidate kernel knows both before it writes
            // the lists; it stores them into pinned host memory and the host polls that word instead of
            // draining the stream, so the bitmap kernel and whatever the caller enqueues next keep the GPU busy.
            unsigned long long word = 0;
            if (!wait_for_report(report, ticket, ticket_before, &word)) {
                // no word within the time limit: drain the stream and look again, then read the counters the slow way
                BUILD_TRY(hipStreamSynchronize(st));
                word = __atomic_load_n(report, __ATOMIC_ACQUIRE);
                if ((uint32_t)(word >> 40) != ticket) {
                    if (slot_counters) {
                        BUILD_TRY(hipMemcpy(&word, p.report_copy, sizeof(word), hipMemcpyDeviceToHost));
                        if ((uint32_t)(word >> 40) != ticket) {
                            status = hdt_fail(HDT_ERR_HIP, "hdt_build_layout: the build kernel finished without its report");
                            goto fail;
                        }
                    } else {
                        int32_t cnt[4] = {0, 0, 0, 0};
                        BUILD_TRY(hipMemcpy(cnt, p.counters, sizeof(cnt), hipMemcpyDeviceToHost));
                        word = report_word(ticket, cnt[CNT_ERR], (uint32_t)cnt[CNT_CAND]);  // low word of the combined counter
                    }
                }
            }
            if ((word >> 39) & 1u) {
                BUILD_TRY(hipStreamSynchronize(st));  // the bitmap kernel still reads the arenas
                status = hdt_fail(HDT_ERR_HIERARCHY, "hdt_build_layout: %s", kHierarchyText);
                goto fail;
            }
            const int64_t need = (int64_t)(word & 0xffffffffu);
            {
                std::lock_guard<std::mutex> lk(g_pool_mutex);
                if (!force_dense) g_capacity_hint = need;
            }
            if (need <= cap) {
                adopt(q, cap);
                L->n_entries = need;
                L->entries_needed = need;
                *out = L;
                return HDT_OK;
            }
            BUILD_TRY(hipStreamSynchronize(st));  // the bitmap kernel still writes the arrays about to be replaced
            if (capacity_opt > 0) {
                status = hdt_fail(HDT_ERR_SHAPE, "hdt_build_layout: the schedule needs %lld list entries, opts->capacity is %lld",
                                  (long long)need, (long long)capacity_opt);
                goto fail;
            }
            // the guess was too small: once more with the exact size
            pool_free(L->arena2, L->arena2_bytes, L->device, only_stream(st));
            L->arena2 = nullptr;
            cap = need;
        }
        status = hdt_fail(HDT_ERR_HIP, "hdt_build_layout: candidate count changed between two passes");
    }
fail:
    hdt_layout_release(L, only_stream((hipStream_t)stream));
    L->magic = 0;
    delete L;
    return status;
#undef BUILD_TRY
}
