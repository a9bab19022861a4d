// hdt_attn_bwd, bf16 MFMA kernels for gfx950.
//
// The paper gives no backward pass; these kernels evaluate the gradient of the definition in
// Sec. 3.2 (S = softmax(mask(Q K^T * scale)), O = S V) over the same surviving tiles the forward
// walks:  D_i = sum_c dO_ic O_ic,  P = exp(S - LSE),  dV = P^T dO,  dP = dO V^T,
//         dS = P o (dP - D),  dQ = scale dS K,  dK = scale dS^T Q.
//
// Two deterministic passes, no atomics:
//   k_bwd_dq   query-major, same shape as the forward kernel: a workgroup owns a query tile, walks
//              its key tiles, recomputes S^T and dP^T with queries along the MFMA columns (so LSE_i
//              and D_i are per-lane scalars) and accumulates dQ^T = K^T dS^T.  It also writes D.
//   k_bwd_dkv  key-major over the transposed lists: a workgroup owns a key tile (64 slots), keeps its
//              K and V rows in registers as MFMA B operands, stages each query tile's Q and dO rows
//              in LDS and accumulates dV^T = dO^T P and dK^T = Q^T dS with keys along the columns.
// Both recompute the scores, which costs two extra contractions but keeps dQ out of HBM as
// fp32 partial sums.
#include "hdt_internal.h"
#include "hdt_mfma.h"

namespace {

constexpr int BM = 128, BN = 64, THREADS = 256;
constexpr float LOG2E = 1.4426950408889634f;

// ------------------------------------------------------------------------------------------- dQ
template <int D>
__global__ __launch_bounds__(THREADS) void k_bwd_dq_bf16(HdtSchedule s, const __bf16 *__restrict__ q,
                                                         const __bf16 *__restrict__ k,
                                                         const __bf16 *__restrict__ v,
                                                         const __bf16 *__restrict__ o,
                                                         const float *__restrict__ lse,
                                                         const __bf16 *__restrict__ d_o, __bf16 *__restrict__ dq,
                                                         float *__restrict__ delta, int heads, float scale)
{
    constexpr int KSTEPS = D / 16, DBLK = D / 32, CPR = D / 8;
    constexpr int NLD = BN * CPR / THREADS, RPP = THREADS / CPR;
    constexpr int K_STRIDE = D * 2 + 32;  // K is read by rows and transposed
    constexpr int V_STRIDE = D * 2 + 16;  // V is read by rows only
    __shared__ __attribute__((aligned(16))) char smem[BN * (K_STRIDE + V_STRIDE)];
    char *sK = smem, *sV = smem + BN * K_STRIDE;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int qn = lane & 31, hf = lane >> 5;
    const int I = blockIdx.x % s.tr, bh = blockIdx.x / s.tr, b = bh / heads;
    const size_t base = (size_t)bh * s.n_pos * D;
    const int32_t *kperm = s.kperm + (size_t)b * s.n_slots;
    const float scale_log2 = scale * LOG2E;

    const int qrow = I * BM + wave * 32 + qn;
    const int qrow_ld = min(qrow, s.n_pos - 1);
    bf16x8 qf[KSTEPS], dof[KSTEPS];
    float Di = 0.f;
#pragma unroll
    for (int st = 0; st < KSTEPS; st++) {
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

    f32x16 dqacc[DBLK];
#pragma unroll
    for (int i = 0; i < DBLK; i++)
#pragma unroll
        for (int e = 0; e < 16; e++) dqacc[i][e] = 0.f;

    const size_t row = (size_t)b * s.tr + I;
    const int t0 = s.q_rowptr[row], t1 = s.q_rowptr[row + 1];
    uint4 kreg[NLD], vreg[NLD];
    const int ld_row = tid / CPR, ld_ch = tid % CPR;
    auto issue_loads = [&](int t) {
        const int J = s.q_cols[t];
#pragma unroll
        for (int p = 0; p < NLD; p++) {
            int pos = kperm[J * BN + ld_row + p * RPP];
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
            *reinterpret_cast<uint4 *>(sK + r * K_STRIDE + ld_ch * 16) = kreg[p];
            *reinterpret_cast<uint4 *>(sV + r * V_STRIDE + ld_ch * 16) = vreg[p];
        }
        __syncthreads();
        if (t + 1 < t1) issue_loads(t + 1);

#pragma unroll
        for (int kb = 0; kb < 2; kb++) {
            const int sb = wave * 2 + kb;
            if (!((sub >> sb) & 1u)) continue;
            f32x16 sacc, dpacc;
#pragma unroll
            for (int e = 0; e < 16; e++) sacc[e] = dpacc[e] = 0.f;
            const char *krow = sK + (kb * 32 + qn) * K_STRIDE + hf * 16;
            const char *vrow = sV + (kb * 32 + qn) * V_STRIDE + hf * 16;
#pragma unroll
            for (int st = 0; st < KSTEPS; st++) {
                sacc = mfma_32x32x16(lds_read_8(krow + st * 32), qf[st], sacc);     // S^T  = K Q^T
                dpacc = mfma_32x32x16(lds_read_8(vrow + st * 32), dof[st], dpacc);  // dP^T = V dO^T
            }
            uint32_t word = 0xffffffffu;
            if (!((sub >> (16 + sb)) & 1u))
                word = s.bits[((size_t)bidx * BM + wave * 32 + qn) * 2 + kb] >> (hf * 4);
#pragma unroll
            for (int e = 0; e < 16; e++) {
                const int bit = 8 * (e / 4) + (e % 4);
                float p = fast_exp2(fmaf(sacc[e], scale_log2, -lse2));
                p = ((word >> bit) & 1u) ? p : 0.f;
                sacc[e] = p * (dpacc[e] - Di);  // dS^T
            }
            // dQ^T += K^T dS^T
            const bf16x8 b0 = pack_bf16x8(sacc, 0), b1 = pack_bf16x8(sacc, 8);
            const int g = lane >> 4, tl = lane & 15;
            const char *kbase =
                sK + (kb * 32 + (g >> 1) * 4 + (tl >> 2)) * K_STRIDE + ((g & 1) * 16 + (tl & 3) * 4) * 2;
#pragma unroll
            for (int i = 0; i < DBLK; i++) {
                const char *kp = kbase + i * 64;
                dqacc[i] = mfma_32x32x16(lds_read_tr_8(kp, kp + 8 * K_STRIDE), b0, dqacc[i]);
                dqacc[i] = mfma_32x32x16(lds_read_tr_8(kp + 16 * K_STRIDE, kp + 24 * K_STRIDE), b1, dqacc[i]);
            }
        }
    }

    if (qrow < s.n_pos) {
        __bf16 *orow = dq + base + (size_t)qrow * D;
#pragma unroll
        for (int i = 0; i < DBLK; i++)
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
__global__ __launch_bounds__(THREADS) void k_bwd_dkv_bf16(HdtSchedule s, const __bf16 *__restrict__ q,
                                                          const __bf16 *__restrict__ k,
                                                          const __bf16 *__restrict__ v,
                                                          const float *__restrict__ lse,
                                                          const __bf16 *__restrict__ d_o,
                                                          const float *__restrict__ delta,
                                                          __bf16 *__restrict__ dk, __bf16 *__restrict__ dv,
                                                          int heads, float scale)
{
    constexpr int KSTEPS = D / 16, DBLK = D / 32, CPR = D / 8;
    constexpr int NLD = BM * CPR / THREADS, RPP = THREADS / CPR;
    constexpr int STRIDE = D * 2 + 32;  // Q and dO rows: read by rows and transposed
    constexpr int TILE_BYTES = BM * STRIDE;
    __shared__ __attribute__((aligned(16))) char smem[2 * TILE_BYTES];
    __shared__ __attribute__((aligned(16))) float sLse[BM], sDelta[BM];
    char *sQ = smem, *sDO = smem + TILE_BYTES;
    static_assert(2 * TILE_BYTES >= 2 * 2 * (D / 32) * 16 * 64 * 4, "reduction buffer must fit");

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int kn = lane & 31, hf = lane >> 5;
    const int kb = wave & 1, qh = wave >> 1;
    const int J = blockIdx.x % s.tc, bh = blockIdx.x / s.tc, b = bh / heads;
    const size_t base = (size_t)bh * s.n_pos * D;
    const float scale_log2 = scale * LOG2E;

    const int pos = s.kperm[(size_t)b * s.n_slots + J * BN + kb * 32 + kn];
    const int pos_ld = pos < 0 ? 0 : pos;
    bf16x8 kf[KSTEPS], vf[KSTEPS];
#pragma unroll
    for (int st = 0; st < KSTEPS; st++) {
        const size_t off = base + (size_t)pos_ld * D + st * 16 + hf * 8;
        kf[st] = *reinterpret_cast<const bf16x8 *>(k + off);
        vf[st] = *reinterpret_cast<const bf16x8 *>(v + off);
    }
    f32x16 dkacc[DBLK], dvacc[DBLK];
#pragma unroll
    for (int i = 0; i < DBLK; i++)
#pragma unroll
        for (int e = 0; e < 16; e++) dkacc[i][e] = dvacc[i][e] = 0.f;

    const size_t col = (size_t)b * s.tc + J;
    const int e0 = s.k_colptr[col], e1 = s.k_colptr[col + 1];
    const int ld_row = tid / CPR, ld_ch = tid % CPR;
    const int g = lane >> 4, tl = lane & 15;

    for (int en = e0; en < e1; en++) {
        const int I = s.k_rows[en], t = s.k_tile[en];
        const uint32_t sub = s.q_sub[t];
        const int bidx = s.q_bidx[t];
        __syncthreads();
#pragma unroll
        for (int p = 0; p < NLD; p++) {
            const int r = ld_row + p * RPP;
            const int i = min(I * BM + r, s.n_pos - 1);
            const size_t off = base + (size_t)i * D + ld_ch * 8;
            *reinterpret_cast<uint4 *>(sQ + r * STRIDE + ld_ch * 16) = *reinterpret_cast<const uint4 *>(q + off);
            *reinterpret_cast<uint4 *>(sDO + r * STRIDE + ld_ch * 16) = *reinterpret_cast<const uint4 *>(d_o + off);
        }
        if (tid < BM) {
            const int i = min(I * BM + tid, s.n_pos - 1);
            const float l = lse[(size_t)bh * s.n_pos + i];
            sLse[tid] = (l == -INFINITY) ? 0.f : l * LOG2E;
            sDelta[tid] = delta[(size_t)bh * s.n_pos + i];
        }
        __syncthreads();

#pragma unroll
        for (int qs = 0; qs < 2; qs++) {
            const int rb = qh * 2 + qs;  // 32-row block of the query tile
            const int sb = rb * 2 + kb;
            if (!((sub >> sb) & 1u)) continue;
            const int r0 = rb * 32;
            f32x16 sacc, dpacc;
#pragma unroll
            for (int e = 0; e < 16; e++) sacc[e] = dpacc[e] = 0.f;
            const char *qrow = sQ + (r0 + kn) * STRIDE + hf * 16;
            const char *dorow = sDO + (r0 + kn) * STRIDE + hf * 16;
#pragma unroll
            for (int st = 0; st < KSTEPS; st++) {
                sacc = mfma_32x32x16(lds_read_8(qrow + st * 32), kf[st], sacc);     // S  = Q K^T
                dpacc = mfma_32x32x16(lds_read_8(dorow + st * 32), vf[st], dpacc);  // dP = dO V^T
            }
            uint32_t word = 0xffffffffu;
            if (!((sub >> (16 + sb)) & 1u))
                word = s.bits_t[((size_t)bidx * BN + kb * 32 + kn) * 4 + rb] >> (hf * 4);
            f32x16 pacc;
#pragma unroll
            for (int gq = 0; gq < 4; gq++) {
                const float4 l4 = *reinterpret_cast<const float4 *>(&sLse[r0 + hf * 4 + gq * 8]);
                const float4 d4 = *reinterpret_cast<const float4 *>(&sDelta[r0 + hf * 4 + gq * 8]);
                const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dl[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    const int idx = gq * 4 + e, bit = 8 * gq + e;
                    float p = fast_exp2(fmaf(sacc[idx], scale_log2, -lv[e]));
                    p = ((word >> bit) & 1u) ? p : 0.f;
                    pacc[idx] = p;
                    sacc[idx] = p * (dpacc[idx] - dl[e]);  // dS
                }
            }
            const bf16x8 p0 = pack_bf16x8(pacc, 0), p1 = pack_bf16x8(pacc, 8);
            const bf16x8 s0 = pack_bf16x8(sacc, 0), s1 = pack_bf16x8(sacc, 8);
            const int off = (r0 + (g >> 1) * 4 + (tl >> 2)) * STRIDE + ((g & 1) * 16 + (tl & 3) * 4) * 2;
#pragma unroll
            for (int i = 0; i < DBLK; i++) {
                const char *dp = sDO + off + i * 64;  // dV^T += dO^T P
                dvacc[i] = mfma_32x32x16(lds_read_tr_8(dp, dp + 8 * STRIDE), p0, dvacc[i]);
                dvacc[i] = mfma_32x32x16(lds_read_tr_8(dp + 16 * STRIDE, dp + 24 * STRIDE), p1, dvacc[i]);
                const char *qp = sQ + off + i * 64;  // dK^T += Q^T dS
                dkacc[i] = mfma_32x32x16(lds_read_tr_8(qp, qp + 8 * STRIDE), s0, dkacc[i]);
                dkacc[i] = mfma_32x32x16(lds_read_tr_8(qp + 16 * STRIDE, qp + 24 * STRIDE), s1, dkacc[i]);
            }
        }
    }

    // add the two query halves (waves qh = 1 hand their sums to waves qh = 0) and store
    __syncthreads();
    float *red = reinterpret_cast<float *>(smem);  // [kb][dk|dv][DBLK][16][64]
    if (qh == 1) {
#pragma unroll
        for (int i = 0; i < DBLK; i++)
#pragma unroll
            for (int e = 0; e < 16; e++) {
                red[(((kb * 2 + 0) * DBLK + i) * 16 + e) * 64 + lane] = dkacc[i][e];
                red[(((kb * 2 + 1) * DBLK + i) * 16 + e) * 64 + lane] = dvacc[i][e];
            }
    }
    __syncthreads();
    if (qh == 0 && pos >= 0) {
        __bf16 *dkrow = dk + base + (size_t)pos * D;
        __bf16 *dvrow = dv + base + (size_t)pos * D;
#pragma unroll
        for (int i = 0; i < DBLK; i++)
#pragma unroll
            for (int gq = 0; gq < 4; gq++) {
                bf16x4 wk, wv;
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    const int idx = gq * 4 + e;
                    const float a = dkacc[i][idx] + red[(((kb * 2 + 0) * DBLK + i) * 16 + idx) * 64 + lane];
                    const float c = dvacc[i][idx] + red[(((kb * 2 + 1) * DBLK + i) * 16 + idx) * 64 + lane];
                    wk[e] = (__bf16)(a * scale);
                    wv[e] = (__bf16)c;
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
    dim3 gq((unsigned)((size_t)s.batch * heads * s.tr)), gk((unsigned)((size_t)s.batch * heads * s.tc));
    dim3 block(THREADS);
    {
        HdtTimer t(head_dim == 64 ? "hdt_bwd_dq_bf16_d64" : "hdt_bwd_dq_bf16_d128", st);
        if (head_dim == 64)
            hipLaunchKernelGGL(k_bwd_dq_bf16<64>, gq, block, 0, st, s, Q, K, V, O, lse, DO, (__bf16 *)dq, delta,
                               heads, scale);
        else
            hipLaunchKernelGGL(k_bwd_dq_bf16<128>, gq, block, 0, st, s, Q, K, V, O, lse, DO, (__bf16 *)dq, delta,
                               heads, scale);
    }
    {
        HdtTimer t(head_dim == 64 ? "hdt_bwd_dkv_bf16_d64" : "hdt_bwd_dkv_bf16_d128", st);
        if (head_dim == 64)
            hipLaunchKernelGGL(k_bwd_dkv_bf16<64>, gk, block, 0, st, s, Q, K, V, lse, DO, delta, (__bf16 *)dk,
                               (__bf16 *)dv, heads, scale);
        else
            hipLaunchKernelGGL(k_bwd_dkv_bf16<128>, gk, block, 0, st, s, Q, K, V, lse, DO, delta, (__bf16 *)dk,
                               (__bf16 *)dv, heads, scale);
    }
    HDT_HIP_TRY(hipGetLastError());
    return HDT_OK;
}
