// hdt_attn_fwd, bf16 MFMA kernel for gfx950.
//
// Follows App. A.1, Alg. 1 of the paper (per query tile: loop over its key tiles, mask, online
// softmax, accumulate P V) over the precomputed list of surviving tiles; O and the softmax
// statistics stay in registers until the last tile and are written once.
//
// Work split: one workgroup (4 waves) per (sample, head, query tile of 128 rows); wave w owns
// query rows 32w .. 32w+31.  A key tile is 64 slots of the level-sorted key order, gathered row
// by row through kperm into LDS (coalesced 16-byte loads, one full 128/256-byte row per 8/16
// lanes).  Inside a tile a wave works on 32x32 sub-blocks and skips those the layout marks empty.
//
// The scores are computed transposed, S^T = K Q^T (keys along the MFMA rows, queries along the
// columns): then every lane owns ONE query (column l%32) and 16 of the 32 keys, so the row max and
// row sum of the online softmax are per-lane scalars plus one exchange between the two half-waves,
// the rescaling factor of O^T = V^T P^T is a per-lane scalar too, and the P^T fragment is already
// in the B-operand layout of the second MFMA (see hdt_mfma.h).  V^T fragments come from LDS with
// the transposing read.
#include "hdt_internal.h"
#include "hdt_mfma.h"

namespace {

constexpr int BM = 128, BN = 64, THREADS = 256;

template <int D>
struct FwdSmem {
    static constexpr int K_STRIDE = D * 2 + 16;  // bytes; 16-byte pad: conflict-free 128-bit row reads
    static constexpr int V_STRIDE = D * 2 + 32;  // bytes; 32-byte pad: conflict-free transposing reads
    static constexpr int K_BYTES = BN * K_STRIDE;
    static constexpr int V_BYTES = BN * V_STRIDE;
};

template <int D>
__global__ __launch_bounds__(THREADS) void k_fwd_bf16(HdtSchedule s, const __bf16 *__restrict__ q,
                                                      const __bf16 *__restrict__ k,
                                                      const __bf16 *__restrict__ v, __bf16 *__restrict__ o,
                                                      float *__restrict__ lse, int heads, float scale_log2)
{
    using SM = FwdSmem<D>;
    constexpr int KSTEPS = D / 16;   // MFMA steps of Q K^T
    constexpr int DBLK = D / 32;     // 32-wide column blocks of O
    constexpr int CPR = D / 8;       // 16-byte chunks per row
    constexpr int NLD = BN * CPR / THREADS;  // chunks per thread per operand
    constexpr int RPP = THREADS / CPR;       // rows per load pass

    __shared__ __attribute__((aligned(16))) char smem[SM::K_BYTES + SM::V_BYTES];
    char *sK = smem, *sV = smem + SM::K_BYTES;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int qn = lane & 31, hf = lane >> 5;
    const int I = blockIdx.x % s.tr, bh = blockIdx.x / s.tr, b = bh / heads;
    const size_t base = (size_t)bh * s.n_pos * D;
    const int32_t *kperm = s.kperm + (size_t)b * s.n_slots;

    // this lane's query row (clamped for loads; rows past n_pos are never stored)
    const int qrow = I * BM + wave * 32 + qn;
    const int qrow_ld = min(qrow, s.n_pos - 1);
    bf16x8 qf[KSTEPS];
#pragma unroll
    for (int st = 0; st < KSTEPS; st++)
        qf[st] = *reinterpret_cast<const bf16x8 *>(q + base + (size_t)qrow_ld * D + st * 16 + hf * 8);

    f32x16 oacc[DBLK];
#pragma unroll
    for (int i = 0; i < DBLK; i++)
#pragma unroll
        for (int e = 0; e < 16; e++) oacc[i][e] = 0.f;
    float m_run = -INFINITY, l_part = 0.f;

    const size_t row = (size_t)b * s.tr + I;
    const int t0 = s.q_rowptr[row], t1 = s.q_rowptr[row + 1];

    // staging registers for the next tile
    uint4 kreg[NLD], vreg[NLD];
    const int ld_row = tid / CPR, ld_ch = tid % CPR;
    auto issue_loads = [&](int t) {
        const int J = s.q_cols[t];
#pragma unroll
        for (int p = 0; p < NLD; p++) {
            const int r = ld_row + p * RPP;
            int pos = kperm[J * BN + r];
            pos = pos < 0 ? 0 : pos;
            const size_t off = base + (size_t)pos * D + ld_ch * 8;
            kreg[p] = *reinterpret_cast<const uint4 *>(k + off);
            vreg[p] = *reinterpret_cast<const uint4 *>(v + off);
        }
    };
    if (t0 < t1) issue_loads(t0);

    for (int t = t0; t < t1; t++) {
        const uint32_t sub = s.q_sub[t];
        const int bidx = s.q_bidx[t];
        __syncthreads();
#pragma unroll
        for (int p = 0; p < NLD; p++) {
            const int r = ld_row + p * RPP;
            *reinterpret_cast<uint4 *>(sK + r * SM::K_STRIDE + ld_ch * 16) = kreg[p];
            *reinterpret_cast<uint4 *>(sV + r * SM::V_STRIDE + ld_ch * 16) = vreg[p];
        }
        __syncthreads();
        if (t + 1 < t1) issue_loads(t + 1);

#pragma unroll
        for (int kb = 0; kb < 2; kb++) {
            const int sb = wave * 2 + kb;
            if (!((sub >> sb) & 1u)) continue;  // empty 32x32 sub-block (wave-uniform)

            // S^T sub-block = K[kb*32 .. +32) . Q^T
            f32x16 sacc;
#pragma unroll
            for (int e = 0; e < 16; e++) sacc[e] = 0.f;
            const char *krow = sK + (kb * 32 + qn) * SM::K_STRIDE + hf * 16;
#pragma unroll
            for (int st = 0; st < KSTEPS; st++) sacc = mfma_32x32x16(lds_read_8(krow + st * 32), qf[st], sacc);

            if (!((sub >> (16 + sb)) & 1u)) {  // not all pairs allowed: apply the bitmap
                const uint32_t word =
                    s.bits[((size_t)bidx * BM + wave * 32 + qn) * 2 + kb] >> (hf * 4);
#pragma unroll
                for (int e = 0; e < 16; e++) {
                    const int bit = 8 * (e / 4) + (e % 4);
                    sacc[e] = ((word >> bit) & 1u) ? sacc[e] : -INFINITY;
                }
            }

            // online softmax for this lane's query over its 16 keys (+ the other half-wave's 16)
            float mx = sacc[0];
#pragma unroll
            for (int e = 1; e < 16; e++) mx = fmaxf(mx, sacc[e]);
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m_run, mx * scale_log2);
            const float m_use = (m_new == -INFINITY) ? 0.f : m_new;  // row fully masked so far
            const float alpha = fast_exp2(m_run - m_use);
            float psum = 0.f;
#pragma unroll
            for (int e = 0; e < 16; e++) {
                sacc[e] = fast_exp2(fmaf(sacc[e], scale_log2, -m_use));
                psum += sacc[e];
            }
            l_part = l_part * alpha + psum;
            m_run = m_new;
            if (__any(alpha != 1.f)) {
#pragma unroll
                for (int i = 0; i < DBLK; i++)
#pragma unroll
                    for (int e = 0; e < 16; e++) oacc[i][e] *= alpha;
            }

            // O^T += V^T P^T
            const bf16x8 pb0 = pack_bf16x8(sacc, 0), pb1 = pack_bf16x8(sacc, 8);
            const int g = lane >> 4, tl = lane & 15;
            const char *vbase =
                sV + (kb * 32 + (g >> 1) * 4 + (tl >> 2)) * SM::V_STRIDE + ((g & 1) * 16 + (tl & 3) * 4) * 2;
#pragma unroll
            for (int i = 0; i < DBLK; i++) {
                const char *vp = vbase + i * 64;
                bf16x8 a0 = lds_read_tr_8(vp, vp + 8 * SM::V_STRIDE);
                oacc[i] = mfma_32x32x16(a0, pb0, oacc[i]);
                bf16x8 a1 = lds_read_tr_8(vp + 16 * SM::V_STRIDE, vp + 24 * SM::V_STRIDE);
                oacc[i] = mfma_32x32x16(a1, pb1, oacc[i]);
            }
        }
    }

    // epilogue: O = acc / l, LSE = ln(sum exp) = ln2 * (m + log2 l)
    const float l_tot = l_part + __shfl_xor(l_part, 32);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    if (qrow < s.n_pos) {
        __bf16 *orow = o + base + (size_t)qrow * D;
#pragma unroll
        for (int i = 0; i < DBLK; i++)
#pragma unroll
            for (int gq = 0; gq < 4; gq++) {
                bf16x4 w;
#pragma unroll
                for (int e = 0; e < 4; e++) w[e] = (__bf16)(oacc[i][gq * 4 + e] * inv);
                *reinterpret_cast<bf16x4 *>(orow + i * 32 + hf * 4 + gq * 8) = w;
            }
        if (hf == 0)
            lse[(size_t)bh * s.n_pos + qrow] =
                l_tot > 0.f ? (m_run + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f : -INFINITY;
    }
}

}  // namespace

hdt_status_t hdt_launch_fwd_bf16(const HdtSchedule &s, const void *q, const void *k, const void *v, void *o,
                                 float *lse, int heads, int head_dim, float scale, hipStream_t st)
{
    const float scale_log2 = scale * 1.4426950408889634f;
    dim3 grid((unsigned)((size_t)s.batch * heads * s.tr)), block(THREADS);
    HdtTimer t(head_dim == 64 ? "hdt_fwd_bf16_d64" : "hdt_fwd_bf16_d128", st);
    if (head_dim == 64)
        hipLaunchKernelGGL(k_fwd_bf16<64>, grid, block, 0, st, s, (const __bf16 *)q, (const __bf16 *)k,
                           (const __bf16 *)v, (__bf16 *)o, lse, heads, scale_log2);
    else
        hipLaunchKernelGGL(k_fwd_bf16<128>, grid, block, 0, st, s, (const __bf16 *)q, (const __bf16 *)k,
                           (const __bf16 *)v, (__bf16 *)o, lse, heads, scale_log2);
    HDT_HIP_TRY(hipGetLastError());
    return HDT_OK;
}
