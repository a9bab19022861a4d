// hdt_attn_fwd, bf16 MFMA kernel for gfx950.
//
// Follows App. A.1, Alg. 1 of the paper (per query tile: loop over its key tiles, mask, online
// softmax, accumulate P V) over the precomputed list of surviving tiles; O and the softmax
// statistics stay in registers until the last tile and are written once.
//
// Work split: one workgroup per (sample, head, query tile of BM rows); wave w owns query rows
// 32w .. 32w+31.  A key tile is one list entry of the query tile: BN key positions in level-sorted
// order, gathered row by row straight into LDS (hdt_tile.h).  Inside a tile a wave works on 32x32
// sub-blocks and skips those the layout marks empty.
//
// The scores are computed transposed, S^T = K Q^T (keys along the MFMA rows, queries along the
// columns): then every lane owns ONE query (column l%32) and 16 of the 32 keys, so the row max and
// row sum of the online softmax are per-lane scalars plus one exchange between the two half-waves,
// the rescaling factor of O^T = V^T P^T is a per-lane scalar too, and the P^T fragment is already
// in the B-operand layout of the second MFMA (see hdt_mfma.h).  V^T fragments come from LDS with
// the transposing read.
//
// Online softmax with a lazily updated reference: exponentials are taken relative to a per-row
// reference m_ref that is only raised (and the accumulators rescaled) when the running maximum
// exceeds it by more than 8 in the log2 domain, so P stays below 2^8 and most sub-blocks skip the
// rescaling of O entirely.  The result is the same quantity as Alg. 1's m/l recurrence:
// O = acc / l and LSE = ln2 * (m_ref + log2 l).
#include "hdt_tile.h"

namespace {

using namespace hdt_tile;

template <int D>
struct FwdCfg {
    static constexpr int S = 2;                      // ring stages (LDS at 128 x 64: 36 KB / 68 KB per workgroup)
    static constexpr int WAVES = (D == 64) ? 4 : 2;  // waves per SIMD the register budget allows
};

// One key tile for one wave: its sub-blocks A0 (keys 0..31) and A1 (keys 32..63) of the tile, as selected.
template <int D, bool A0, bool A1>
__device__ __forceinline__ void fwd_step(const char *sK, const char *sV, const RowLane &rl, const TrLane &tl,
                                         const bf16x8 (&qf)[D / 16], f32x16 (&oacc)[D / 32], float &m_ref,
                                         float &l_part, const unsigned long long *mk, int xlane, float scale_log2)
{
    constexpr int ROWB = 2 * D, KSTEPS = D / 16, DBLK = D / 32;
    // S^T sub-blocks = K[kb*32 .. +32) . Q^T, masked
    f32x16 s0, s1;
#pragma unroll
    for (int e = 0; e < 16; e++) s0[e] = s1[e] = 0.f;
#pragma unroll
    for (int st = 0; st < KSTEPS; st++) {
        if (A0) s0 = mfma_32x32x16(read_row<ROWB>(sK, rl, 0, st), qf[st], s0);
        if (A1) s1 = mfma_32x32x16(read_row<ROWB>(sK, rl, 32, st), qf[st], s1);
    }
    float mx = -INFINITY;
    if (A0) {
        apply_mask(s0, mk, -INFINITY);
#pragma unroll
        for (int e = 0; e < 16; e += 2) mx = fmaxf(mx, fmaxf(s0[e], s0[e + 1]));
    }
    if (A1) {
        apply_mask(s1, mk + 16, -INFINITY);
#pragma unroll
        for (int e = 0; e < 16; e += 2) mx = fmaxf(mx, fmaxf(s1[e], s1[e + 1]));
    }

    // online softmax for this lane's query over up to 64 keys: its own registers plus those of
    // the partner lane in the other half-wave
    mx = fmaxf(mx, __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(xlane, __builtin_bit_cast(int, mx))));
    mx *= scale_log2;
    if (__any(mx > m_ref + 8.f)) {  // raise the reference and rescale (always on a row's first keys)
        const float m_new = fmaxf(m_ref, mx);
        const float alpha = (m_new == -INFINITY) ? 1.f : fast_exp2(m_ref - m_new);
        m_ref = m_new;
        l_part *= alpha;
#pragma unroll
        for (int j = 0; j < DBLK; j++)
#pragma unroll
            for (int e = 0; e < 16; e++) oacc[j][e] *= alpha;
    }
    const float m_sub = (m_ref == -INFINITY) ? 0.f : m_ref;  // row without any allowed key so far

    // P^T = exp2(S^T * scale*log2e - m_ref); O^T += V^T P^T
    float psum = 0.f;
    bf16x8 p00, p01, p10, p11;
    if (A0) {
#pragma unroll
        for (int e = 0; e < 16; e++) {
            s0[e] = fast_exp2(fmaf(s0[e], scale_log2, -m_sub));
            psum += s0[e];
        }
        p00 = pack_bf16x8(s0, 0);
        p01 = pack_bf16x8(s0, 8);
    }
    if (A1) {
#pragma unroll
        for (int e = 0; e < 16; e++) {
            s1[e] = fast_exp2(fmaf(s1[e], scale_log2, -m_sub));
            psum += s1[e];
        }
        p10 = pack_bf16x8(s1, 0);
        p11 = pack_bf16x8(s1, 8);
    }
    l_part += psum;
#pragma unroll
    for (int j = 0; j < DBLK; j++) {
        if (A0) {
            oacc[j] = mfma_32x32x16(read_tr<ROWB>(sV, tl, 0, j), p00, oacc[j]);
            oacc[j] = mfma_32x32x16(read_tr<ROWB>(sV, tl, 16, j), p01, oacc[j]);
        }
        if (A1) {
            oacc[j] = mfma_32x32x16(read_tr<ROWB>(sV, tl, 32, j), p10, oacc[j]);
            oacc[j] = mfma_32x32x16(read_tr<ROWB>(sV, tl, 48, j), p11, oacc[j]);
        }
    }
}

template <int D, typename G>
__global__ __launch_bounds__(G::THREADS, FwdCfg<D>::WAVES) void k_fwd_bf16(
    HdtSchedule s, const __bf16 *__restrict__ q, const __bf16 *__restrict__ k, const __bf16 *__restrict__ v,
    __bf16 *__restrict__ o, float *__restrict__ lse, int heads, float scale_log2)
{
    using P = Pipe<D, FwdCfg<D>::S, false, G>;
    using R = Ring<P>;
    constexpr int BM = G::BM, BN = G::BN, KB = G::KB;
    constexpr int ROWB = P::ROWB, KSTEPS = P::KSTEPS, DBLK = P::DBLK, S = P::S;
    __shared__ __attribute__((aligned(1024))) char smem[P::SMEM_BYTES];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int qn = lane & 31, hf = lane >> 5;
    const unsigned lb = logical_block(blockIdx.x, G::XCD_CHUNK);
    if (lb >= (unsigned)s.batch * heads * s.tr) return;  // padding of the grid
    const int I = lb % s.tr, bh = lb / s.tr, b = bh / heads;
    const int I_own = I % s.tr_own;  // the rows this tile works on (several tiles share them when key lists are cut)
    const size_t base = (size_t)bh * s.n_pos * D, own_base = (size_t)bh * s.n_own * D, kv_base = (size_t)bh * s.n_kv * D;

    const size_t row = (size_t)b * s.tr + I;
    const cptr_i32 range = as_const(s.q_range);
    const int t0 = range[2 * row], n = range[2 * row + 1] - t0;
    const cptr_u32 subs = as_const(s.q_sub) + t0;

    P pipe;
    pipe.smem = smem;
    pipe.smem_addr = lds_addr(smem);
    pipe.wave = wave;
    pipe.lane = lane;
    pipe.keys = s.q_keys + (size_t)t0 * BN;
    pipe.a = k + kv_base;
    pipe.b = v + kv_base;
    pipe.aux0 = pipe.aux1 = nullptr;
    // this lane's query row; rows past n_pos are computed on a clamped copy and never stored
    const int qrow = I * BM + wave * 32 + qn;
    const RowLane rl = row_lane<P::CPR>(lane);
    const TrLane tl = tr_lane<P::CPR>(lane);

    // Q rows of this wave go through the ring stage the prologue leaves free (S-1): full-row loads
    // into LDS, then the B fragments (query l%32, 8 head-dim values per step) are read back
    constexpr uint32_t Q_STAGE = (uint32_t)(S - 1) * 2 * P::TILE;
    bf16x8 qf[KSTEPS];
    if (n > 0) {
        stage_own_rows(pipe, q + own_base, I_own * BM, s.n_own, D, Q_STAGE);
        R::start(pipe, n);
        R::template prologue<0, S - 1>(pipe, n);  // its first wait covers the Q rows
#pragma unroll
        for (int st = 0; st < KSTEPS; st++) qf[st] = read_row<ROWB>(smem + Q_STAGE, rl, wave * 32, st);
    }

    f32x16 oacc[DBLK];
#pragma unroll
    for (int i = 0; i < DBLK; i++)
#pragma unroll
        for (int e = 0; e < 16; e++) oacc[i][e] = 0.f;
    float m_ref = -INFINITY, l_part = 0.f;
    const int xlane = (lane ^ 32) << 2;  // ds_bpermute address of the partner lane in the other half-wave

    uint32_t sub_next = n > 0 ? subs[0] : 0u;
    for (int i = 0; i < n; i++) {
        const uint32_t sub = sub_next;
        const int bidx = t0 + i;  // bitmaps are stored in list order
        if (i + 1 < n) {
            sub_next = subs[i + 1];
        }
        R::top(i, n);
        wg_barrier();
        R::advance(pipe, i, n);
        const char *sK = pipe.tile_a(i % S), *sV = pipe.tile_b(i % S);

        // this wave's two 32x32 sub-blocks of the tile (wave-uniform flags); one straight-line code path
        // per combination, so that the two sub-blocks' loads, MFMA chains and exponentials interleave
        const bool act0 = (sub >> (wave * KB)) & 1u, act1 = KB > 1 && ((sub >> (wave * KB + 1)) & 1u);
        if (!(act0 || act1)) continue;
        const unsigned long long *mk = s.bits_rm + ((size_t)bidx * G::NSUB + wave * KB) * 16;
        if (KB > 1 && act0 && act1)
            fwd_step<D, true, true>(sK, sV, rl, tl, qf, oacc, m_ref, l_part, mk, xlane, scale_log2);
        else if (act0)
            fwd_step<D, true, false>(sK, sV, rl, tl, qf, oacc, m_ref, l_part, mk, xlane, scale_log2);
        else if (KB > 1)
            fwd_step<D, false, true>(sK, sV, rl, tl, qf, oacc, m_ref, l_part, mk, xlane, scale_log2);
    }

    // epilogue: O = acc / l, LSE = ln(sum exp) = ln2 * (m_ref + log2 l); O leaves through LDS as full rows
    const float l_tot = l_part + __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(xlane, __builtin_bit_cast(int, l_part)));
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    // The rows leave through this wave's slice of the ring stage that tile n would have used: nothing was
    // loaded into it after tile n - S, which every wave finished reading before the last barrier (for the
    // first S tiles: only each wave's own staged rows), so no barrier is needed and a wave that is done
    // early does not wait for the others.
    const int wrow0 = I * BM + wave * 32;
    store_rows_via_lds<P, D>(smem + (n % S) * 2 * P::TILE + wave * 32 * ROWB, lane, oacc, inv,
                             o + base + (size_t)wrow0 * D, s.n_pos - wrow0);
    if (qrow < s.n_pos && hf == 0)
        lse[(size_t)bh * s.n_pos + qrow] = l_tot > 0.f ? (m_ref + __builtin_amdgcn_logf(l_tot)) * LN2 : -INFINITY;
}

}  // namespace

template <typename G>
static void launch_fwd(const HdtSchedule &s, const void *q, const void *k, const void *v, void *o, float *lse,
                       int heads, int head_dim, float scale_log2, hipStream_t st)
{
    dim3 grid(padded_grid((unsigned)((size_t)s.batch * heads * s.tr), G::XCD_CHUNK)), block(G::THREADS);
    if (head_dim == 64)
        hipLaunchKernelGGL((k_fwd_bf16<64, G>), grid, block, 0, st, s, (const __bf16 *)q, (const __bf16 *)k,
                           (const __bf16 *)v, (__bf16 *)o, lse, heads, scale_log2);
    else
        hipLaunchKernelGGL((k_fwd_bf16<128, G>), grid, block, 0, st, s, (const __bf16 *)q, (const __bf16 *)k,
                           (const __bf16 *)v, (__bf16 *)o, lse, heads, scale_log2);
}

hdt_status_t hdt_launch_fwd_bf16(const HdtSchedule &s, const void *q, const void *k, const void *v, void *o,
                                 float *lse, int heads, int head_dim, float scale, hipStream_t st)
{
    const float scale_log2 = scale * LOG2E;
    HdtTimer t(head_dim == 64 ? "hdt_fwd_bf16_d64" : "hdt_fwd_bf16_d128", st);
    if (s.bm == 64)
        launch_fwd<Geo<64, 32>>(s, q, k, v, o, lse, heads, head_dim, scale_log2, st);
    else
        launch_fwd<Geo<128, 64>>(s, q, k, v, o, lse, heads, head_dim, scale_log2, st);
    HDT_HIP_TRY(hipGetLastError());
    return HDT_OK;
}
