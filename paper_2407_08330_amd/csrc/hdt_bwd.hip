// hdt_attn_bwd, bf16 MFMA kernels for gfx950.
//
// The paper gives no backward pass; these kernels evaluate the gradient of the definition in
// Sec. 3.2 (S = softmax(mask(Q K^T * scale)), O = S V) over the same surviving tiles the forward
// walks:  D_i = sum_c dO_ic O_ic,  P = exp(S - LSE),  dV = P^T dO,  dP = dO V^T,
//         dS = P o (dP - D),  dQ = scale dS K,  dK = scale dS^T Q.
//
// Two deterministic passes, no atomics, both with the forward kernel's skeleton (hdt_tile.h):
//   k_bwd_dq   a workgroup owns a query tile (rows in document order), walks its key tiles (slots of
//              the level-sorted order, gathered through kperm), recomputes S^T and dP^T with queries
//              along the MFMA columns (LSE_i and D_i are per-lane scalars) and accumulates
//              dQ^T = K^T dS^T.  It also writes D.
//   k_bwd_dkv  the mask is symmetric (i may attend to j iff j may attend to i: parent/child and
//              sibling relations are mutual), so the tile list of "query rows I x key slots J" is also
//              the list of "key rows I x query slots J", bitmaps included.  A workgroup therefore owns
//              128 KEYS in document order (K, V rows in registers), walks the same list, gathers the
//              Q and dO rows (and LSE, D) of 64 level-sorted QUERY slots into LDS and accumulates
//              dV^T = dO^T P and dK^T = Q^T dS with keys along the MFMA columns.  Same load balance
//              as the forward, no transposed lists, no cross-wave reduction, contiguous stores.
// Both passes recompute the scores, which costs two extra contractions but keeps dQ out of HBM
// as fp32 partial sums.
#include "hdt_tile.h"

namespace {

using namespace hdt_tile;

// ------------------------------------------------------------------------------------------- dQ
template <int D>
__global__ __launch_bounds__(THREADS, 2) void k_bwd_dq_bf16(HdtSchedule s, const __bf16 *__restrict__ q,
                                                            const __bf16 *__restrict__ k,
                                                            const __bf16 *__restrict__ v,
                                                            const __bf16 *__restrict__ o,
                                                            const float *__restrict__ lse,
                                                            const __bf16 *__restrict__ d_o,
                                                            __bf16 *__restrict__ dq, float *__restrict__ delta,
                                                            int heads, float scale)
{
    using G = Geom<D>;
    constexpr int K_STRIDE = G::TR_STRIDE;   // K is read by rows and transposed
    constexpr int V_STRIDE = G::ROW_STRIDE;  // V is read by rows only
    __shared__ __attribute__((aligned(16))) char smem[BN * (K_STRIDE + V_STRIDE)];
    char *sK = smem, *sV = smem + BN * K_STRIDE;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int qn = lane & 31, hf = lane >> 5;
    const unsigned lb = logical_block(blockIdx.x, gridDim.x);
    const int I = lb % s.tr, bh = lb / s.tr, b = bh / heads;
    const size_t base = (size_t)bh * s.n_pos * D;
    const int32_t *kperm = s.kperm + (size_t)b * s.n_slots;
    const float scale_log2 = scale * LOG2E;

    const size_t row = (size_t)b * s.tr + I;
    const int t0 = s.q_rowptr[row], t1 = s.q_rowptr[row + 1];
    Entry e0 = load_entry(s, t0, t1), e1 = load_entry(s, t0 + 1, t1), e2 = load_entry(s, t0 + 2, t1);

    const int qrow = I * BM + wave * 32 + qn;
    const int qrow_ld = min(qrow, s.n_pos - 1);
    bf16x8 qf[G::KSTEPS], dof[G::KSTEPS];
    float Di = 0.f;
#pragma unroll
    for (int st = 0; st < G::KSTEPS; st++) {
        const size_t off = base + (size_t)qrow_ld * D + st * 16 + hf * 8;
        qf[st] = *reinterpret_cast<const bf16x8 *>(q + off);
        dof[st] = *reinterpret_cast<const bf16x8 *>(d_o + off);
        const bf16x8 of = *reinterpret_cast<const bf16x8 *>(o + off);
#pragma unroll
        for (int e = 0; e < 8; e++) Di += (float)dof[st][e] * (float)of[e];
    }
    Di += __shfl_xor(Di, 32);
    if (qrow < s.n_pos && hf == 0) delta[(size_t)bh * s.n_pos + qrow] = Di;
    float lse2 = lse[(size_t)bh * s.n_pos + qrow_ld];
    lse2 = (lse2 == -INFINITY) ? 0.f : lse2 * LOG2E;  // pad rows are masked by the bitmap anyway

    f32x16 dqacc[G::DBLK];
#pragma unroll
    for (int i = 0; i < G::DBLK; i++)
#pragma unroll
        for (int e = 0; e < 16; e++) dqacc[i][e] = 0.f;

    const int ld_row = tid / G::CPR, ld_ch = tid % G::CPR;
    int pos1[G::NLD], pos2[G::NLD];
    u32x4 kreg[G::NLD], vreg[G::NLD];
#pragma unroll
    for (int p = 0; p < G::NLD; p++) pos1[p] = pos2[p] = 0;
    if (t0 < t1) {
        load_positions<D>(kperm, e0.col, ld_row, pos1);
        if (t0 + 1 < t1) load_positions<D>(kperm, e1.col, ld_row, pos2);
        gather_rows<D>(k, v, base, pos1, ld_ch, kreg, vreg);
#pragma unroll
        for (int p = 0; p < G::NLD; p++) pos1[p] = pos2[p];
    }
    const int ktr = tr_offset(lane, K_STRIDE);

    for (int t = t0; t < t1; t++) {
        __syncthreads();
        stage_rows<D, K_STRIDE, V_STRIDE>(sK, sV, ld_row, ld_ch, kreg, vreg);
        __syncthreads();
        if (t + 1 < t1) gather_rows<D>(k, v, base, pos1, ld_ch, kreg, vreg);
        if (t + 2 < t1) load_positions<D>(kperm, e2.col, ld_row, pos1);
        const Entry e3 = load_entry(s, t + 3, t1);

#pragma unroll
        for (int kb = 0; kb < 2; kb++) {
            const int sb = wave * 2 + kb;
            if (!((e0.sub >> sb) & 1u)) continue;
            f32x16 sacc, dpacc;
#pragma unroll
            for (int e = 0; e < 16; e++) sacc[e] = dpacc[e] = 0.f;
            const char *krow = sK + (kb * 32 + qn) * K_STRIDE + hf * 16;
            const char *vrow = sV + (kb * 32 + qn) * V_STRIDE + hf * 16;
#pragma unroll
            for (int st = 0; st < G::KSTEPS; st++) {
                sacc = mfma_32x32x16(lds_read_8(krow + st * 32), qf[st], sacc);     // S^T  = K Q^T
                dpacc = mfma_32x32x16(lds_read_8(vrow + st * 32), dof[st], dpacc);  // dP^T = V dO^T
            }
#pragma unroll
            for (int e = 0; e < 16; e++) sacc[e] = fast_exp2(fmaf(sacc[e], scale_log2, -lse2));  // P^T
            if (!((e0.sub >> (16 + sb)) & 1u))
                apply_mask(sacc, s.bits_rm + ((size_t)e0.bidx * 8 + sb) * 16, 0.f);
#pragma unroll
            for (int e = 0; e < 16; e++) sacc[e] *= dpacc[e] - Di;  // dS^T
            // dQ^T += K^T dS^T
            const bf16x8 b0 = pack_bf16x8(sacc, 0), b1 = pack_bf16x8(sacc, 8);
            const char *kbase = sK + kb * 32 * K_STRIDE + ktr;
#pragma unroll
            for (int i = 0; i < G::DBLK; i++) {
                const char *kp = kbase + i * 64;
                dqacc[i] = mfma_32x32x16(lds_read_tr_8(kp, kp + 8 * K_STRIDE), b0, dqacc[i]);
                dqacc[i] = mfma_32x32x16(lds_read_tr_8(kp + 16 * K_STRIDE, kp + 24 * K_STRIDE), b1, dqacc[i]);
            }
        }
        e0 = e1;
        e1 = e2;
        e2 = e3;
    }

    if (qrow < s.n_pos) {
        __bf16 *orow = dq + base + (size_t)qrow * D;
#pragma unroll
        for (int i = 0; i < G::DBLK; i++)
#pragma unroll
            for (int gq = 0; gq < 4; gq++) {
                bf16x4 w;
#pragma unroll
                for (int e = 0; e < 4; e++) w[e] = (__bf16)(dqacc[i][gq * 4 + e] * scale);
                *reinterpret_cast<bf16x4 *>(orow + i * 32 + hf * 4 + gq * 8) = w;
            }
    }
}

// ---------------------------------------------------------------------------------------- dK, dV
template <int D>
__global__ __launch_bounds__(THREADS, (D == 64 ? 2 : 1)) void k_bwd_dkv_bf16(
    HdtSchedule s, const __bf16 *__restrict__ q, const __bf16 *__restrict__ k, const __bf16 *__restrict__ v,
    const float *__restrict__ lse, const __bf16 *__restrict__ d_o, const float *__restrict__ delta,
    __bf16 *__restrict__ dk, __bf16 *__restrict__ dv, int heads, float scale)
{
    using G = Geom<D>;
    constexpr int STRIDE = G::TR_STRIDE;  // Q and dO tiles: read by rows and transposed
    __shared__ __attribute__((aligned(16))) char smem[2 * BN * STRIDE];
    __shared__ __attribute__((aligned(16))) float sAux[2 * BN];  // LSE*log2e and D of the 64 query slots
    char *sQ = smem, *sDO = smem + BN * STRIDE;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kn = lane & 31, hf = lane >> 5;
    const unsigned lb = logical_block(blockIdx.x, gridDim.x);
    const int I = lb % s.tr, bh = lb / s.tr, b = bh / heads;
    const size_t base = (size_t)bh * s.n_pos * D;
    const size_t vbase = (size_t)bh * s.n_pos;
    const int32_t *kperm = s.kperm + (size_t)b * s.n_slots;
    const float scale_log2 = scale * LOG2E;

    const size_t row = (size_t)b * s.tr + I;
    const int t0 = s.q_rowptr[row], t1 = s.q_rowptr[row + 1];
    Entry e0 = load_entry(s, t0, t1), e1 = load_entry(s, t0 + 1, t1), e2 = load_entry(s, t0 + 2, t1);

    // this lane's key row, document order
    const int krow = I * BM + wave * 32 + kn;
    const int krow_ld = min(krow, s.n_pos - 1);
    bf16x8 kf[G::KSTEPS], vf[G::KSTEPS];
#pragma unroll
    for (int st = 0; st < G::KSTEPS; st++) {
        const size_t off = base + (size_t)krow_ld * D + st * 16 + hf * 8;
        kf[st] = *reinterpret_cast<const bf16x8 *>(k + off);
        vf[st] = *reinterpret_cast<const bf16x8 *>(v + off);
    }
    f32x16 dkacc[G::DBLK], dvacc[G::DBLK];
#pragma unroll
    for (int i = 0; i < G::DBLK; i++)
#pragma unroll
        for (int e = 0; e < 16; e++) dkacc[i][e] = dvacc[i][e] = 0.f;

    const int ld_row = tid / G::CPR, ld_ch = tid % G::CPR;
    int pos1[G::NLD], pos2[G::NLD];
    u32x4 qreg[G::NLD], doreg[G::NLD];
    // threads 0..63 fetch LSE of slot tid, threads 64..127 fetch D of slot tid-64
    const float *aux_src = (tid < BN) ? lse : delta;
    const int aux_slot = tid & (BN - 1);
    int apos1 = 0, apos2 = 0;
    float aux_reg = 0.f;
#pragma unroll
    for (int p = 0; p < G::NLD; p++) pos1[p] = pos2[p] = 0;
    if (t0 < t1) {
        load_positions<D>(kperm, e0.col, ld_row, pos1);
        apos1 = max(kperm[e0.col * BN + aux_slot], 0);
        if (t0 + 1 < t1) {
            load_positions<D>(kperm, e1.col, ld_row, pos2);
            apos2 = max(kperm[e1.col * BN + aux_slot], 0);
        }
        gather_rows<D>(q, d_o, base, pos1, ld_ch, qreg, doreg);
        if (tid < 2 * BN) aux_reg = aux_src[vbase + apos1];
#pragma unroll
        for (int p = 0; p < G::NLD; p++) pos1[p] = pos2[p];
        apos1 = apos2;
    }
    const int tro = tr_offset(lane, STRIDE);

    for (int t = t0; t < t1; t++) {
        __syncthreads();
        stage_rows<D, STRIDE, STRIDE>(sQ, sDO, ld_row, ld_ch, qreg, doreg);
        if (tid < BN)
            sAux[tid] = (aux_reg == -INFINITY) ? 0.f : aux_reg * LOG2E;
        else if (tid < 2 * BN)
            sAux[tid] = aux_reg;
        __syncthreads();
        if (t + 1 < t1) {
            gather_rows<D>(q, d_o, base, pos1, ld_ch, qreg, doreg);
            if (tid < 2 * BN) aux_reg = aux_src[vbase + apos1];
        }
        if (t + 2 < t1) {
            load_positions<D>(kperm, e2.col, ld_row, pos1);
            apos1 = max(kperm[e2.col * BN + aux_slot], 0);
        }
        const Entry e3 = load_entry(s, t + 3, t1);

#pragma unroll
        for (int kb = 0; kb < 2; kb++) {  // 32 query slots
            const int sb = wave * 2 + kb;
            if (!((e0.sub >> sb) & 1u)) continue;
            f32x16 sacc, dpacc;
#pragma unroll
            for (int e = 0; e < 16; e++) sacc[e] = dpacc[e] = 0.f;
            const char *qrow = sQ + (kb * 32 + kn) * STRIDE + hf * 16;
            const char *dorow = sDO + (kb * 32 + kn) * STRIDE + hf * 16;
#pragma unroll
            for (int st = 0; st < G::KSTEPS; st++) {
                sacc = mfma_32x32x16(lds_read_8(qrow + st * 32), kf[st], sacc);     // S  = Q K^T
                dpacc = mfma_32x32x16(lds_read_8(dorow + st * 32), vf[st], dpacc);  // dP = dO V^T
            }
            f32x16 pacc;
#pragma unroll
            for (int gq = 0; gq < 4; gq++) {
                const float4 l4 = *reinterpret_cast<const float4 *>(&sAux[kb * 32 + hf * 4 + gq * 8]);
                const float lv[4] = {l4.x, l4.y, l4.z, l4.w};
#pragma unroll
                for (int e = 0; e < 4; e++)
                    pacc[gq * 4 + e] = fast_exp2(fmaf(sacc[gq * 4 + e], scale_log2, -lv[e]));
            }
            if (!((e0.sub >> (16 + sb)) & 1u))
                apply_mask(pacc, s.bits_rm + ((size_t)e0.bidx * 8 + sb) * 16, 0.f);
#pragma unroll
            for (int gq = 0; gq < 4; gq++) {
                const float4 d4 = *reinterpret_cast<const float4 *>(&sAux[BN + kb * 32 + hf * 4 + gq * 8]);
                const float dl[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
                for (int e = 0; e < 4; e++) sacc[gq * 4 + e] = pacc[gq * 4 + e] * (dpacc[gq * 4 + e] - dl[e]);  // dS
            }
            const bf16x8 p0 = pack_bf16x8(pacc, 0), p1 = pack_bf16x8(pacc, 8);
            const bf16x8 s0 = pack_bf16x8(sacc, 0), s1 = pack_bf16x8(sacc, 8);
            const int off = kb * 32 * STRIDE + tro;
#pragma unroll
            for (int i = 0; i < G::DBLK; i++) {
                const char *dp = sDO + off + i * 64;  // dV^T += dO^T P
                dvacc[i] = mfma_32x32x16(lds_read_tr_8(dp, dp + 8 * STRIDE), p0, dvacc[i]);
                dvacc[i] = mfma_32x32x16(lds_read_tr_8(dp + 16 * STRIDE, dp + 24 * STRIDE), p1, dvacc[i]);
                const char *qp = sQ + off + i * 64;  // dK^T += Q^T dS
                dkacc[i] = mfma_32x32x16(lds_read_tr_8(qp, qp + 8 * STRIDE), s0, dkacc[i]);
                dkacc[i] = mfma_32x32x16(lds_read_tr_8(qp + 16 * STRIDE, qp + 24 * STRIDE), s1, dkacc[i]);
            }
        }
        e0 = e1;
        e1 = e2;
        e2 = e3;
    }

    if (krow < s.n_pos) {
        __bf16 *dkrow = dk + base + (size_t)krow * D;
        __bf16 *dvrow = dv + base + (size_t)krow * D;
#pragma unroll
        for (int i = 0; i < G::DBLK; i++)
#pragma unroll
            for (int gq = 0; gq < 4; gq++) {
                bf16x4 wk, wv;
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    wk[e] = (__bf16)(dkacc[i][gq * 4 + e] * scale);
                    wv[e] = (__bf16)dvacc[i][gq * 4 + e];
                }
                *reinterpret_cast<bf16x4 *>(dkrow + i * 32 + hf * 4 + gq * 8) = wk;
                *reinterpret_cast<bf16x4 *>(dvrow + i * 32 + hf * 4 + gq * 8) = wv;
            }
    }
}

}  // namespace

hdt_status_t hdt_launch_bwd_bf16(const HdtSchedule &s, const void *q, const void *k, const void *v,
                                 const void *o, const float *lse, const void *d_o, void *dq, void *dk, void *dv,
                                 int heads, int head_dim, float scale, float *delta, hipStream_t st)
{
    const __bf16 *Q = (const __bf16 *)q, *K = (const __bf16 *)k, *V = (const __bf16 *)v;
    const __bf16 *O = (const __bf16 *)o, *DO = (const __bf16 *)d_o;
    dim3 grid((unsigned)((size_t)s.batch * heads * s.tr)), block(THREADS);
    {
        HdtTimer t(head_dim == 64 ? "hdt_bwd_dq_bf16_d64" : "hdt_bwd_dq_bf16_d128", st);
        if (head_dim == 64)
            hipLaunchKernelGGL(k_bwd_dq_bf16<64>, grid, block, 0, st, s, Q, K, V, O, lse, DO, (__bf16 *)dq, delta,
                               heads, scale);
        else
            hipLaunchKernelGGL(k_bwd_dq_bf16<128>, grid, block, 0, st, s, Q, K, V, O, lse, DO, (__bf16 *)dq, delta,
                               heads, scale);
    }
    {
        HdtTimer t(head_dim == 64 ? "hdt_bwd_dkv_bf16_d64" : "hdt_bwd_dkv_bf16_d128", st);
        if (head_dim == 64)
            hipLaunchKernelGGL(k_bwd_dkv_bf16<64>, grid, block, 0, st, s, Q, K, V, lse, DO, delta, (__bf16 *)dk,
                               (__bf16 *)dv, heads, scale);
        else
            hipLaunchKernelGGL(k_bwd_dkv_bf16<128>, grid, block, 0, st, s, Q, K, V, lse, DO, delta, (__bf16 *)dk,
                               (__bf16 *)dv, heads, scale);
    }
    HDT_HIP_TRY(hipGetLastError());
    return HDT_OK;
}
