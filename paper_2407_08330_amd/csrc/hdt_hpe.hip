// Hierarchical positional encoding (paper Sec. 3.2 "Hierarchical Positional Encoding", Eq. pos_enc,
// Fig. 3 caption): every position carries one index per hierarchy level, each index goes through the
// standard sinusoidal functions, and the encodings of the levels are summed and added to the embeddings.
//
//   hdt_parents_from_levels  levels of a document in the paper's layout (anchors in front) -> parent ids
//   hdt_index_vectors   level/parent ids -> index vectors p[B][N][L] (1-based ordinal among the siblings
//                       of the position's ancestor-or-self at each level, 0 where there is none)
//   hdt_hpe_table       the sinusoidal table T[v][c] = sin / cos (w_k v), w_k = 10000^(-2k/d_model)
//   hdt_hpe_add         x[b][n][c] += sum_l T[p^l][c]
//
// The indices of a document are small integers (ordinal of a section, of a sentence in its section, of a
// token in its sentence), so the encoding of a position is the sum of L rows of a small table that stays in
// L2: the add is then bound by reading and writing x once, not by 2*L*d_model sine evaluations per position.
// Indices beyond the table are evaluated directly.
#include <math.h>

#include "hdt_internal.h"

namespace {

constexpr int kOrdThreads = 1024, kOrdWaves = kOrdThreads / 64;

// ---- parents of a document laid out with its anchors in front (pre-order) ---------------------------
// parent[i] = the nearest earlier position whose level is level[i] - 1 (none: -1).  One workgroup per
// sample walks the positions in chunks of 1024 and keeps, per level, the last position seen so far:
// inside a wave by ballots, across the waves of a chunk and across chunks through LDS.
__global__ __launch_bounds__(kOrdThreads) void k_parents_from_levels(const int32_t *__restrict__ level, int n,
                                                                      int32_t *__restrict__ parent)
{
    __shared__ int s_last[kOrdWaves][32];  // last position of each level in each wave of the chunk (-1: none)
    __shared__ int s_carry[32];            // last position of each level in the chunks before
    const int b = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const size_t o = (size_t)b * n;
    if (tid < 32) s_carry[tid] = -1;
    __syncthreads();
    for (int c0 = 0; c0 < n; c0 += kOrdThreads) {
        const int i = c0 + tid;
        int lv = i < n ? level[o + i] : -1;
        if (lv < 0 || lv >= 32) lv = -1;
        // the last lane of every level in this wave, kept by lane = level
        int mine = -1;
        for (int l = 0; l < 32; l++) {
            const unsigned long long m = __ballot(lv == l);
            if (lane == l && m) mine = c0 + wave * 64 + 63 - __builtin_clzll(m);
        }
        if (lane < 32) s_last[wave][lane] = mine;
        // the nearest earlier lane of this wave with level lv - 1
        int par = -1;
        unsigned long long todo = __ballot(lv > 0);
        while (todo) {
            const int leader = __ffsll((long long)todo) - 1;
            const int t = __builtin_amdgcn_readlane(lv, leader) - 1;
            const unsigned long long m = __ballot(lv == t);
            const bool me = lv - 1 == t && lv > 0;
            const unsigned long long before = m & ((1ull << lane) - 1ull);
            if (me && before) par = c0 + wave * 64 + 63 - __builtin_clzll(before);
            todo &= ~__ballot(me);
        }
        __syncthreads();
        if (lv > 0 && par < 0) {  // not in this wave: earlier waves of the chunk, then earlier chunks
            for (int w = wave - 1; w >= 0 && par < 0; w--) par = s_last[w][lv - 1];
            if (par < 0) par = s_carry[lv - 1];
        }
        if (i < n) parent[o + i] = par;
        __syncthreads();
        if (tid < 32) {
            for (int w = kOrdWaves - 1; w >= 0; w--)
                if (s_last[w][tid] >= 0) {
                    s_carry[tid] = s_last[w][tid];
                    break;
                }
        }
        __syncthreads();
    }
}

// ---- ordinal of every position among its siblings (same parent), in document order ---------------
// One workgroup per sample walks the positions in chunks of 1024 * kOrdV (a thread takes kOrdV consecutive
// positions).  Inside a chunk, consecutive positions with the same parent form a run (the tokens of a sentence,
// for one): a position's ordinal is
//   1 + (siblings in earlier chunks: a per-parent counter in global memory)
//     + (siblings in earlier runs of this chunk: a sum over the earlier run heads, shared by kOrdSplit lanes)
//     + (its offset inside its run).
// Roots (parent -1) count as children of one virtual parent.  Pads and positions past n form runs of
// their own (group -1), which only serve to end the runs before them.
constexpr int kOrdV = 4, kOrdChunk = kOrdThreads * kOrdV, kOrdSplit = 16;

__global__ __launch_bounds__(kOrdThreads) void k_sibling_ordinals(const int32_t *__restrict__ level,
                                                                   const int32_t *__restrict__ parent, int n,
                                                                   int32_t *cnt,  // [B][n + 1] scratch
                                                                   int32_t *ord)  // [B][n]
{
    // per run head of the chunk: its group, its first position in the chunk; per position of the chunk that
    // starts a run: siblings before that run (s_run_base)
    __shared__ int s_head_parent[kOrdChunk], s_head_start[kOrdChunk], s_run_base[kOrdChunk];
    __shared__ int s_last_grp[kOrdThreads];
    __shared__ int s_wave_max[kOrdWaves], s_wave_heads[kOrdWaves];
    const int b = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const size_t o = (size_t)b * n;
    int32_t *my_cnt = cnt + (size_t)b * (n + 1);
    for (int i = tid; i <= n; i += kOrdThreads) my_cnt[i] = 0;
    __syncthreads();
    for (int c0 = 0; c0 < n; c0 += kOrdChunk) {
        const int idx0 = tid * kOrdV;  // this thread's first position inside the chunk
        int grp[kOrdV];                // the parent (n for roots), -1 for pads and positions past n
#pragma unroll
        for (int u = 0; u < kOrdV; u++) {
            const int i = c0 + idx0 + u;
            grp[u] = -1;
            if (i < n && level[o + i] >= 0) {
                const int p = parent[o + i];
                grp[u] = (p >= 0 && p < n) ? p : n;
            }
        }
        s_last_grp[tid] = grp[kOrdV - 1];
        __syncthreads();
        // run heads; the last head at or before every position: a running maximum over the threads
        int before = tid == 0 ? -2 : s_last_grp[tid - 1];
        bool head[kOrdV];
        int n_mine = 0, last_head = -1;
#pragma unroll
        for (int u = 0; u < kOrdV; u++) {
            head[u] = grp[u] != before;
            before = grp[u];
            if (head[u]) {
                n_mine++;
                last_head = idx0 + u;
            }
        }
        int run_max = last_head, heads_incl = n_mine;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int y = __shfl_up(run_max, d), z = __shfl_up(heads_incl, d);
            if (lane >= d) {
                run_max = max(run_max, y);
                heads_incl += z;
            }
        }
        if (lane == 63) {
            s_wave_max[wave] = run_max;
            s_wave_heads[wave] = heads_incl;
        }
        __syncthreads();
        int start_in = __shfl_up(run_max, 1);  // last head before this thread's positions
        if (lane == 0) start_in = -1;
        int my_head = heads_incl - n_mine, n_heads = 0;
        for (int w = 0; w < kOrdWaves; w++) {
            if (w < wave) {
                start_in = max(start_in, s_wave_max[w]);
                my_head += s_wave_heads[w];
            }
            n_heads += s_wave_heads[w];
        }
        int start[kOrdV];
        {
            int cur = start_in, h = my_head;
#pragma unroll
            for (int u = 0; u < kOrdV; u++) {
                if (head[u]) {
                    cur = idx0 + u;
                    s_head_parent[h] = grp[u];
                    s_head_start[h] = cur;
                    h++;
                }
                start[u] = cur;
            }
        }
        __syncthreads();
        // siblings in earlier runs of this chunk: kOrdSplit lanes share the scan over the earlier heads of one head
        for (int h = tid / kOrdSplit; h < n_heads; h += kOrdThreads / kOrdSplit) {
            const int g = s_head_parent[h];
            if (g < 0) continue;
            int k = 0;
            for (int e = tid % kOrdSplit; e < h; e += kOrdSplit)
                if (s_head_parent[e] == g) k += s_head_start[e + 1] - s_head_start[e];
#pragma unroll
            for (int d = 1; d < kOrdSplit; d <<= 1) k += __shfl_xor(k, d);
            if (tid % kOrdSplit == 0) {
                // siblings in earlier chunks (the counter last changed before the barrier that ended the previous chunk)
                const int base = __hip_atomic_load(&my_cnt[g], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                s_run_base[s_head_start[h]] = base + k;
            }
        }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < kOrdV; u++)
            if (grp[u] >= 0) ord[o + c0 + idx0 + u] = 1 + s_run_base[start[u]] + (idx0 + u - start[u]);
        // add this chunk's runs to the counters; the returned value makes the thread wait for the atomic
        {
            int h = my_head;
#pragma unroll
            for (int u = 0; u < kOrdV; u++) {
                if (!head[u]) continue;
                if (grp[u] >= 0) {
                    const int end = h + 1 < n_heads ? s_head_start[h + 1] : kOrdChunk;
                    const int old = atomicAdd(&my_cnt[grp[u]], end - (idx0 + u));
                    asm volatile("" ::"v"(old));
                }
                h++;
            }
        }
        __syncthreads();
    }
}

// ---- index vectors: walk up the ancestors ------------------------------------------------------------
__global__ __launch_bounds__(256) void k_index_vectors(const int32_t *__restrict__ level,
                                                       const int32_t *__restrict__ parent,
                                                       const int32_t *__restrict__ ord, int n, int L, int64_t total,
                                                       int32_t *__restrict__ p)
{
    const int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= total) return;
    const int64_t b = g / n;
    const int i = (int)(g - b * n);
    const size_t o = (size_t)b * n;
    int32_t *mine = p + (size_t)g * L;
    for (int l = 0; l < L; l++) mine[l] = 0;
    if (level[o + i] < 0) return;
    int a = i;
    for (int steps = 0; a >= 0 && a < n && steps < 2 * HDT_MAX_LEVELS; steps++) {
        const int l = level[o + a];
        if (l < 0) break;
        if (l >= 1 && l <= L) mine[l - 1] = ord[o + a];
        a = parent[o + a];
    }
}

// ---- the sinusoidal table ------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_hpe_table(float *__restrict__ table, int rows, int d_model)
{
    const int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= (int64_t)rows * d_model) return;
    const int v = (int)(g / d_model), c = (int)(g - (int64_t)v * d_model);
    const double w = pow(10000.0, -2.0 * (double)(c / 2) / (double)d_model);
    const double x = w * (double)v;
    table[g] = (float)((c & 1) ? cos(x) : sin(x));
}

// ---- x += sum over the levels of the table rows -------------------------------------------------------
// A thread owns 8 consecutive channels (16 bytes of bf16) of kPerThread consecutive positions (neighbouring
// positions mostly share their upper-level indices, so their table rows come out of the vector cache); the
// index vectors of its positions are read first, then all table rows and x values are requested together,
// then everything is added and stored: the kernel is a stream over x with the table rows coming out of L2.
// (Measured at d_model 768 / 1024, 32768 positions: 1 position per thread 23.0 / 29.7 us, 2: 24.0 / 29.6,
// 4: 27.1 / 34.3, 8: 40.3 / 48.7; positions a quarter of the tensor apart instead of consecutive: 1-2 us more.)
constexpr int kPerThread = 2, kMaxLevelsFast = 8;

__device__ __noinline__ float hpe_direct(int v, int c, int d_model)
{
    const double w = pow(10000.0, -2.0 * (double)(c / 2) / (double)d_model);
    const double x = w * (double)v;
    return (float)((c & 1) ? cos(x) : sin(x));
}

template <bool BF16>
__global__ __launch_bounds__(256) void k_hpe_add(const int32_t *__restrict__ p, unsigned positions, int L,
                                                 const float *__restrict__ table, int rows, void *__restrict__ x,
                                                 int d_model, unsigned pos_stride)
{
    typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
    const unsigned per_pos = (unsigned)d_model / 8u;
    const unsigned g = blockIdx.x * blockDim.x + threadIdx.x;  // (position inside the quarter, channel group)
    const unsigned pos0 = g / per_pos, c0 = (g - pos0 * per_pos) * 8u;
    if (pos0 >= pos_stride) return;
#define POS(u) (pos0 * kPerThread + (u))
    float acc[kPerThread][8];
    bool live[kPerThread];
#pragma unroll
    for (int u = 0; u < kPerThread; u++) {
        live[u] = POS(u) < positions;
#pragma unroll
        for (int e = 0; e < 8; e++) acc[u][e] = 0.f;
    }
    for (int l0 = 0; l0 < L; l0 += kMaxLevelsFast) {
        int v[kPerThread][kMaxLevelsFast];
#pragma unroll
        for (int u = 0; u < kPerThread; u++)
#pragma unroll
            for (int l = 0; l < kMaxLevelsFast; l++)
                v[u][l] = (live[u] && l0 + l < L) ? p[(size_t)POS(u) * L + l0 + l] : -1;
#pragma unroll
        for (int u = 0; u < kPerThread; u++)
#pragma unroll
            for (int l = 0; l < kMaxLevelsFast; l++) {
                if (l0 + l >= L || !live[u]) continue;
                const int vv = v[u][l];
                if (vv >= 0 && vv < rows) {
                    const float4 t0 = *reinterpret_cast<const float4 *>(table + (size_t)vv * d_model + c0);
                    const float4 t1 = *reinterpret_cast<const float4 *>(table + (size_t)vv * d_model + c0 + 4);
                    acc[u][0] += t0.x, acc[u][1] += t0.y, acc[u][2] += t0.z, acc[u][3] += t0.w;
                    acc[u][4] += t1.x, acc[u][5] += t1.y, acc[u][6] += t1.z, acc[u][7] += t1.w;
                } else {
                    for (int e = 0; e < 8; e++) acc[u][e] += hpe_direct(vv, (int)c0 + e, d_model);
                }
            }
    }
#pragma unroll
    for (int u = 0; u < kPerThread; u++) {
        if (!live[u]) continue;
        const size_t at = (size_t)POS(u) * per_pos + c0 / 8u;
        if (BF16) {
            bf16x8 *px = reinterpret_cast<bf16x8 *>(x) + at;
            bf16x8 val = *px;
#pragma unroll
            for (int e = 0; e < 8; e++) val[e] = (__bf16)((float)val[e] + acc[u][e]);
            *px = val;
        } else {
            float4 *px = reinterpret_cast<float4 *>(x) + 2 * at;
            float4 a = px[0], c = px[1];
            a.x += acc[u][0], a.y += acc[u][1], a.z += acc[u][2], a.w += acc[u][3];
            c.x += acc[u][4], c.y += acc[u][5], c.z += acc[u][6], c.w += acc[u][7];
            px[0] = a;
            px[1] = c;
        }
    }
}

}  // namespace

extern "C" __attribute__((visibility("default"))) hdt_status_t hdt_parents_from_levels(const int32_t *d_level,
                                                                                        int32_t batch, int32_t n_pos,
                                                                                        int32_t *d_parent, void *stream)
{
    if (batch < 0 || n_pos < 0) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_parents_from_levels: negative size");
    if (batch == 0 || n_pos == 0) return HDT_OK;
    if (!d_level || !d_parent) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_parents_from_levels: NULL pointer");
    if ((int64_t)batch * n_pos > (1LL << 30)) return hdt_fail(HDT_ERR_SHAPE, "hdt_parents_from_levels: batch * n_pos too large");
    hipStream_t st = (hipStream_t)stream;
    HdtTimer t("hdt_hpe_parents_from_levels", st);
    hipLaunchKernelGGL(k_parents_from_levels, dim3((unsigned)batch), dim3(kOrdThreads), 0, st, d_level, n_pos, d_parent);
    HDT_HIP_TRY(hipGetLastError());
    return HDT_OK;
}

extern "C" __attribute__((visibility("default"))) size_t hdt_index_vectors_workspace_bytes(int32_t batch, int32_t n_pos)
{
    if (batch <= 0 || n_pos <= 0) return 0;
    // per-parent counters [B][N+1] and sibling ordinals [B][N]
    const size_t ints = (size_t)batch * ((size_t)n_pos + 1) + (size_t)batch * (size_t)n_pos;
    return (ints * sizeof(int32_t) + 255) & ~(size_t)255;
}

extern "C" __attribute__((visibility("default"))) hdt_status_t hdt_index_vectors(
    const int32_t *d_level, const int32_t *d_parent, int32_t batch, int32_t n_pos, int32_t n_levels, int32_t *d_p,
    void *workspace, size_t workspace_bytes, void *stream)
{
    if (batch < 0 || n_pos < 0) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_index_vectors: negative size");
    if (n_levels < 1 || n_levels >= HDT_MAX_LEVELS)
        return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_index_vectors: n_levels = %d (1 .. %d)", n_levels, HDT_MAX_LEVELS - 1);
    if (batch == 0 || n_pos == 0) return HDT_OK;
    if (!d_level || !d_parent || !d_p) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_index_vectors: NULL pointer");
    const size_t need = hdt_index_vectors_workspace_bytes(batch, n_pos);
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 15u))
        return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_index_vectors: workspace of %zu bytes (16-byte aligned) needed", need);
    if ((int64_t)batch * n_pos > (1LL << 30)) return hdt_fail(HDT_ERR_SHAPE, "hdt_index_vectors: batch * n_pos too large");
    hipStream_t st = (hipStream_t)stream;
    int32_t *cnt = static_cast<int32_t *>(workspace);
    int32_t *ord = cnt + (size_t)batch * ((size_t)n_pos + 1);
    {
        HdtTimer t("hdt_hpe_sibling_ordinals", st);
        hipLaunchKernelGGL(k_sibling_ordinals, dim3((unsigned)batch), dim3(kOrdThreads), 0, st, d_level, d_parent,
                           n_pos, cnt, ord);
    }
    {
        const int64_t total = (int64_t)batch * n_pos;
        HdtTimer t("hdt_hpe_index_vectors", st);
        hipLaunchKernelGGL(k_index_vectors, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, d_level, d_parent,
                           ord, n_pos, n_levels, total, d_p);
    }
    HDT_HIP_TRY(hipGetLastError());
    return HDT_OK;
}

extern "C" __attribute__((visibility("default"))) hdt_status_t hdt_hpe_table(float *d_table, int32_t rows,
                                                                              int32_t d_model, void *stream)
{
    if (rows < 0 || d_model <= 0 || d_model % 8) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_hpe_table: rows >= 0, d_model a positive multiple of 8");
    if (rows == 0) return HDT_OK;
    if (!d_table || ((uintptr_t)d_table & 15u)) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_hpe_table: NULL or misaligned table");
    const int64_t total = (int64_t)rows * d_model;
    if (total > (1LL << 31)) return hdt_fail(HDT_ERR_SHAPE, "hdt_hpe_table: table too large");
    HdtTimer t("hdt_hpe_table", (hipStream_t)stream);
    hipLaunchKernelGGL(k_hpe_table, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, (hipStream_t)stream, d_table,
                       rows, d_model);
    HDT_HIP_TRY(hipGetLastError());
    return HDT_OK;
}

extern "C" __attribute__((visibility("default"))) hdt_status_t hdt_hpe_add(const int32_t *d_p, int32_t batch,
                                                                            int32_t n_pos, int32_t n_levels,
                                                                            const float *d_table, int32_t table_rows,
                                                                            void *x, int32_t d_model, hdt_dtype_t dt,
                                                                            void *stream)
{
    if (batch < 0 || n_pos < 0 || table_rows < 0) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_hpe_add: negative size");
    if (n_levels < 1 || n_levels >= HDT_MAX_LEVELS) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_hpe_add: n_levels = %d", n_levels);
    if (d_model <= 0 || d_model % 8) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_hpe_add: d_model must be a positive multiple of 8");
    if (dt != HDT_BF16 && dt != HDT_F32) return hdt_fail(HDT_ERR_UNSUPPORTED, "hdt_hpe_add: unknown dtype %d", (int)dt);
    if (batch == 0 || n_pos == 0) return HDT_OK;
    if (!d_p || !x || (table_rows > 0 && !d_table)) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_hpe_add: NULL pointer");
    if (((uintptr_t)x & 15u) || ((uintptr_t)d_table & 15u)) return hdt_fail(HDT_ERR_INVALID_ARG, "hdt_hpe_add: pointers must be 16-byte aligned");
    const int64_t positions = (int64_t)batch * n_pos;
    const int64_t pos_stride = (positions + kPerThread - 1) / kPerThread, threads = pos_stride * (d_model / 8);
    if (positions > 0x7fffffffLL || threads > 0x7fffffffLL) return hdt_fail(HDT_ERR_SHAPE, "hdt_hpe_add: too many elements");
    hipStream_t st = (hipStream_t)stream;
    HdtTimer t(dt == HDT_BF16 ? "hdt_hpe_add_bf16" : "hdt_hpe_add_f32", st);
    if (dt == HDT_BF16)
        hipLaunchKernelGGL(k_hpe_add<true>, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, d_p,
                           (unsigned)positions, n_levels, d_table, table_rows, x, d_model, (unsigned)pos_stride);
    else
        hipLaunchKernelGGL(k_hpe_add<false>, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, d_p,
                           (unsigned)positions, n_levels, d_table, table_rows, x, d_model, (unsigned)pos_stride);
    HDT_HIP_TRY(hipGetLastError());
    return HDT_OK;
}
