// fp32 debugging path: the same tile schedule walked with plain fp32 arithmetic, one thread per
// query row (forward, dQ) or per key row (dK, dV).  Slow on purpose; it exists to check the
// schedule, the mask bitmaps and the online softmax separately from the MFMA kernels.
// Forward: App. A.1, Alg. 1 (online softmax over the surviving tiles).  Backward: gradient of
// the definition in Sec. 3.2.
#include "hdt_internal.h"

namespace {

template <int D>
__global__ __launch_bounds__(128) void k_fwd_f32(HdtSchedule s, const float *__restrict__ q,
                                                 const float *__restrict__ k, const float *__restrict__ v,
                                                 float *__restrict__ o, float *__restrict__ lse, int heads,
                                                 float scale)
{
    const int I = blockIdx.x, bh = blockIdx.y, b = bh / heads, r = threadIdx.x;
    if (r >= s.bm) return;
    const int i = I * s.bm + r;
    if (i >= s.n_pos) return;
    const size_t base = (size_t)bh * s.n_pos * D, kv_base = (size_t)bh * s.n_kv * D;
    const float *qi = q + base + (size_t)i * D;
    float acc[D];
    for (int c = 0; c < D; c++) acc[c] = 0.f;
    float m = -INFINITY, l = 0.f;
    const size_t row = (size_t)b * s.tr + I;
    for (int t = s.q_range[2 * row]; t < s.q_range[2 * row + 1]; t++) {
        for (int c = 0; c < s.bn; c++) {
            if (!hdt_pair_allowed(s.bits_rm, s.bm, s.wpr, (size_t)t, r, c)) continue;
            const int pos = s.q_keys[(size_t)t * s.bn + c];
            if (pos < 0) continue;
            const float *kj = k + kv_base + (size_t)pos * D;
            const float *vj = v + kv_base + (size_t)pos * D;
            float sc = 0.f;
            for (int e = 0; e < D; e++) sc += qi[e] * kj[e];
            sc *= scale;
            const float m_new = fmaxf(m, sc);
            const float alpha = expf(m - m_new);  // m = -inf -> 0
            const float p = expf(sc - m_new);
            l = l * alpha + p;
            for (int e = 0; e < D; e++) acc[e] = acc[e] * alpha + p * vj[e];
            m = m_new;
        }
    }
    float *oi = o + base + (size_t)i * D;
    const float inv = l > 0.f ? 1.f / l : 0.f;
    for (int c = 0; c < D; c++) oi[c] = acc[c] * inv;
    lse[(size_t)bh * s.n_pos + i] = l > 0.f ? m + logf(l) : -INFINITY;
}

template <int D>
__global__ __launch_bounds__(128) void k_bwd_dq_f32(HdtSchedule s, const float *__restrict__ q,
                                                    const float *__restrict__ k, const float *__restrict__ v,
                                                    const float *__restrict__ o, const float *__restrict__ lse,
                                                    const float *__restrict__ d_o, float *__restrict__ dq,
                                                    float *__restrict__ delta, int heads, float scale)
{
    const int I = blockIdx.x, bh = blockIdx.y, b = bh / heads, r = threadIdx.x;
    if (r >= s.bm) return;
    const int i = I * s.bm + r;
    if (i >= s.n_pos) return;
    const size_t base = (size_t)bh * s.n_pos * D, kv_base = (size_t)bh * s.n_kv * D;
    const float *qi = q + base + (size_t)i * D;
    const float *doi = d_o + base + (size_t)i * D;
    const float *oi = o + base + (size_t)i * D;
    float Di = 0.f;
    for (int c = 0; c < D; c++) Di += doi[c] * oi[c];
    delta[(size_t)bh * s.n_pos + i] = Di;
    const float li = lse[(size_t)bh * s.n_pos + i];
    float acc[D];
    for (int c = 0; c < D; c++) acc[c] = 0.f;
    const size_t row = (size_t)b * s.tr + I;
    for (int t = s.q_range[2 * row]; t < s.q_range[2 * row + 1]; t++) {
        for (int c = 0; c < s.bn; c++) {
            if (!hdt_pair_allowed(s.bits_rm, s.bm, s.wpr, (size_t)t, r, c)) continue;
            const int pos = s.q_keys[(size_t)t * s.bn + c];
            if (pos < 0) continue;
            const float *kj = k + kv_base + (size_t)pos * D;
            const float *vj = v + kv_base + (size_t)pos * D;
            float sc = 0.f, dp = 0.f;
            for (int e = 0; e < D; e++) {
                sc += qi[e] * kj[e];
                dp += doi[e] * vj[e];
            }
            const float p = expf(sc * scale - li);
            const float ds = p * (dp - Di) * scale;
            for (int e = 0; e < D; e++) acc[e] += ds * kj[e];
        }
    }
    float *dqi = dq + base + (size_t)i * D;
    for (int c = 0; c < D; c++) dqi[c] = acc[c];
}

// dK, dV: walks the schedule of the transposed mask (for the paper's symmetric mask that is the forward's
// own schedule: the list of query tile I x key slots J is also the list of key rows I x query slots J with
// the same bitmaps; directed variants bring a second schedule).  One thread per
// key row (document order) walks that list and gathers the query rows its entries name.
template <int D>
__global__ __launch_bounds__(128) void k_bwd_dkv_f32(HdtSchedule s, const float *__restrict__ q,
                                                     const float *__restrict__ k, const float *__restrict__ v,
                                                     const float *__restrict__ lse, const float *__restrict__ d_o,
                                                     const float *__restrict__ delta, float *__restrict__ dk,
                                                     float *__restrict__ dv, int heads, float scale)
{
    const int I = blockIdx.x, bh = blockIdx.y, b = bh / heads, r = threadIdx.x;
    if (r >= s.bm) return;
    const int j = I * s.bm + r;  // key position
    if (j >= s.n_pos) return;
    const size_t base = (size_t)bh * s.n_pos * D, q_base = (size_t)bh * s.n_kv * D;  // rows are keys here
    const float *kj = k + base + (size_t)j * D;
    const float *vj = v + base + (size_t)j * D;
    float ak[D], av[D];
    for (int e = 0; e < D; e++) ak[e] = av[e] = 0.f;
    const size_t row = (size_t)b * s.tr + I;
    for (int t = s.q_range[2 * row]; t < s.q_range[2 * row + 1]; t++) {
        for (int c = 0; c < s.bn; c++) {
            if (!hdt_pair_allowed(s.bits_rm, s.bm, s.wpr, (size_t)t, r, c)) continue;
            const int i = s.q_keys[(size_t)t * s.bn + c];  // query position
            if (i < 0) continue;
            const float *qi = q + q_base + (size_t)i * D;
            const float *doi = d_o + q_base + (size_t)i * D;
            float sc = 0.f, dp = 0.f;
            for (int e = 0; e < D; e++) {
                sc += qi[e] * kj[e];
                dp += doi[e] * vj[e];
            }
            const float p = expf(sc * scale - lse[(size_t)bh * s.n_kv + i]);
            const float ds = p * (dp - delta[(size_t)bh * s.n_kv + i]) * scale;
            for (int e = 0; e < D; e++) {
                av[e] += p * doi[e];
                ak[e] += ds * qi[e];
            }
        }
    }
    float *dkj = dk + base + (size_t)j * D;
    float *dvj = dv + base + (size_t)j * D;
    for (int e = 0; e < D; e++) {
        dkj[e] = ak[e];
        dvj[e] = av[e];
    }
}

}  // namespace

hdt_status_t hdt_launch_fwd_f32(const HdtSchedule &s, const float *q, const float *k, const float *v, float *o,
                                float *lse, int heads, int head_dim, float scale, hipStream_t st)
{
    if ((int64_t)s.batch * heads > 65535) return hdt_fail(HDT_ERR_SHAPE, "fp32 path: batch*heads > 65535");
    dim3 grid(s.tr, s.batch * heads), block(128);
    HdtTimer t("hdt_fwd_f32", st);
    if (head_dim == 64)
        hipLaunchKernelGGL(k_fwd_f32<64>, grid, block, 0, st, s, q, k, v, o, lse, heads, scale);
    else
        hipLaunchKernelGGL(k_fwd_f32<128>, grid, block, 0, st, s, q, k, v, o, lse, heads, scale);
    HDT_HIP_TRY(hipGetLastError());
    return HDT_OK;
}

hdt_status_t hdt_launch_bwd_f32(const HdtSchedule &s, const HdtSchedule &st_, const float *q, const float *k, const float *v,
                                const float *o, const float *lse, const float *d_o, float *dq, float *dk,
                                float *dv, int heads, int head_dim, float scale, float *delta, hipStream_t st)
{
    if ((int64_t)s.batch * heads > 65535) return hdt_fail(HDT_ERR_SHAPE, "fp32 path: batch*heads > 65535");
    dim3 gq(s.tr, s.batch * heads), gk(st_.tr, s.batch * heads), block(128);
    {
        HdtTimer t("hdt_bwd_dq_f32", st);
        if (head_dim == 64)
            hipLaunchKernelGGL(k_bwd_dq_f32<64>, gq, block, 0, st, s, q, k, v, o, lse, d_o, dq, delta, heads, scale);
        else
            hipLaunchKernelGGL(k_bwd_dq_f32<128>, gq, block, 0, st, s, q, k, v, o, lse, d_o, dq, delta, heads, scale);
    }
    {
        HdtTimer t("hdt_bwd_dkv_f32", st);
        if (head_dim == 64)
            hipLaunchKernelGGL(k_bwd_dkv_f32<64>, gk, block, 0, st, st_, q, k, v, lse, d_o, delta, dk, dv, heads, scale);
        else
            hipLaunchKernelGGL(k_bwd_dkv_f32<128>, gk, block, 0, st, st_, q, k, v, lse, d_o, delta, dk, dv, heads, scale);
    }
    HDT_HIP_TRY(hipGetLastError());
    return HDT_OK;
}
