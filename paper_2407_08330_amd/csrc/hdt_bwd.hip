// hdt_attn_bwd, bf16 MFMA kernels for gfx950.
//
// The paper gives no backward pass; these kernels evaluate the gradient of the definition in
// Sec. 3.2 (S = softmax(mask(Q K^T * scale)), O = S V) over the same surviving tiles the forward
// walks:  D_i = sum_c dO_ic O_ic,  P = exp(S - LSE),  dV = P^T dO,  dP = dO V^T,
//         dS = P o (dP - D),  dQ = scale dS K,  dK = scale dS^T Q.
//
// Deterministic, no atomics.  Two launches:
//   k_bwd_delta  D for every row (a streaming pass over O and dO).
//   k_bwd_bf16   two workgroups per row tile I (rows in document order), one per role, both with the
//                forward kernel's skeleton (hdt_tile.h):
//     dQ role      the tile's rows as QUERIES: walks their key tiles (the key positions of each list
//                  entry, gathered row by row), recomputes S^T and dP^T with queries along the MFMA
//                  columns (LSE_i and D_i are per-lane scalars) and accumulates dQ^T = K^T dS^T.
//     dK/dV role   the tile's rows as KEYS: walks the schedule of the TRANSPOSED mask.  The paper's mask
//                  is symmetric (i may attend to j iff j may attend to i: parent/child and sibling
//                  relations are mutual), so the entries of "query rows I x the keys they attend to" are
//                  also the entries of "key rows I x the queries attending to them", bitmaps included.
//                  K, V rows of the tile sit in registers; the Q and dO rows (and LSE, D) of an entry's
//                  QUERY positions are gathered into LDS and dV^T = dO^T P, dK^T = Q^T dS accumulate
//                  with keys along the MFMA columns.  Same load balance as the forward, no cross-wave
//                  reduction, contiguous stores.  For the directed variants (edge kinds without up/down
//                  symmetry) the layout holds a second schedule, built from the same ids with the
//                  parent and child kinds exchanged.
// Both roles recompute the scores, which costs two extra contractions but keeps dQ out of HBM as fp32
// partial sums.  At head size 128 the dK/dV role is split once more, into a dV role and a dK role (three
// workgroups per tile): together they would need more registers than two waves per SIMD leave.  The two workgroups of a tile are neighbours in the launch order and run on the same XCD
// at the same time.  That is what the pairing is for: the dQ role reads the tile's Q, dO rows and gathers
// K, V rows of the neighbourhood, the dK/dV role reads the tile's K, V rows and gathers Q, dO rows of the
// same neighbourhood, so each role finds in the XCD's L2 what the other (or a neighbouring pair) has just
// fetched, and Q, K, V, dO come from HBM once per backward pass instead of once per role (measured: the
// L2 fetch volume of this kernel is that of four tensors; as two separate passes it was that of eight).
#include "hdt_tile.h"

namespace {

using namespace hdt_tile;

template <int D>
struct BwdCfg {
    // ring stages of the two roles and waves per SIMD (register budget) of the kernel.  Three waves at head size
    // 64 pay on 128 x 64 tiles only (measured, config 4: 107 us against 122 with two; on 64 x 32 tiles 101
    // against 99 with two, whose allocation the compiler then leaves unconstrained).
    static constexpr int S_DQ = (D == 64) ? 3 : 2;
    static constexpr int S_DKV = 2;
    template <typename G>
    static constexpr int WAVES = (D == 64 && G::BM == 128) ? 3 : 2;
    // At head size 128 the dK/dV role would need 128 accumulator registers per lane on top of 64 operand
    // registers, which leaves one wave per SIMD.  It is split there into a dV role and a dK role (each
    // recomputes the scores), so that every role fits two waves per SIMD.
    static constexpr bool SPLIT_KV = D == 128;
};

// ---------------------------------------------------------------------------------------- D
// For all rows of [rows][D] tensors: D_i = sum_c dO_ic O_ic (every lane multiplies 8 values, 16 bytes of each
// tensor; the lanes of a row are added up; kRows rows per lane in flight).  What the main kernel wants of a row
// are the two values its contractions start from, so those are what is written, side by side:
//   .x = -D_i            dP - D        = -D + dO V^T          (accumulator of dP preset to it)
//   .y = -LSE_i / scale  scale S - LSE = scale (-LSE / scale + Q K^T)   (accumulator of S preset to it)
// which takes a subtraction and a multiplication per score out of both roles.  Rows without a key (LSE = -inf:
// pads) get 0 for both: they are masked, and their dO may hold anything.
template <int D>
__global__ __launch_bounds__(256) void k_bwd_delta(const __bf16 *__restrict__ o, const __bf16 *__restrict__ d_o,
                                                   const float *__restrict__ lse, float inv_scale,
                                                   float2 *__restrict__ row_scalars, long long rows)
{
    constexpr int CPR = D / 8, RPB = 256 / CPR, kRows = 4;
    const int lr = threadIdx.x / CPR, c = threadIdx.x % CPR;
    const long long r0 = (long long)blockIdx.x * (RPB * kRows) + lr;
    bf16x8 a[kRows], b[kRows];
    float l[kRows];
#pragma unroll
    for (int u = 0; u < kRows; u++) {
        const long long r = min(r0 + (long long)u * RPB, rows - 1);
        a[u] = *reinterpret_cast<const bf16x8 *>(o + (size_t)r * D + c * 8);
        b[u] = *reinterpret_cast<const bf16x8 *>(d_o + (size_t)r * D + c * 8);
        l[u] = c == 0 ? lse[r] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < kRows; u++) {
        float part = 0.f;
#pragma unroll
        for (int e = 0; e < 8; e++) part += (float)a[u][e] * (float)b[u][e];
#pragma unroll
        for (int m = 1; m < CPR; m <<= 1) part += __shfl_xor(part, m);
        const long long r = r0 + (long long)u * RPB;
        if (c == 0 && r < rows) {
            const bool dead = l[u] == -INFINITY;
            row_scalars[r] = dead ? make_float2(0.f, 0.f) : make_float2(-part, -l[u] * inv_scale);
        }
    }
}

// ------------------------------------------------------------------------------------------- dQ
template <int D, typename G>
__device__ __forceinline__ void dq_role(char *smem, const HdtSchedule &s, const __bf16 *__restrict__ q,
                                         const __bf16 *__restrict__ k, const __bf16 *__restrict__ v,
                                         const float *__restrict__ lse, const __bf16 *__restrict__ d_o,
                                         const float2 *__restrict__ row_scalars, __bf16 *__restrict__ dq, int wave,
                                         int I, int bh, int b, float scale)
{
    using P = Pipe<D, BwdCfg<D>::S_DQ, false, G>;
    using R = Ring<P>;
    constexpr int BM = G::BM, BN = G::BN, KB = G::KB;
    constexpr int ROWB = P::ROWB, KSTEPS = P::KSTEPS, DBLK = P::DBLK, S = P::S;

    const int lane = threadIdx.x & 63;
    const int qn = lane & 31;
    const int I_own = I % s.tr_own;  // the rows this tile works on (several tiles share them when key lists are cut)
    const size_t base = (size_t)bh * s.n_pos * D, own_base = (size_t)bh * s.n_own * D, kv_base = (size_t)bh * s.n_kv * D;
    const float scale_log2 = scale * LOG2E;

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
    const int qrow = I_own * BM + wave * 32 + qn;
    const RowLane rl = row_lane<P::CPR>(lane);
    const TrLane tl = tr_lane<P::CPR>(lane);

    // Q and dO rows of this wave go through the two highest ring stages (full-row loads into LDS);
    // the B fragments are read back from there.  The ring may only take those stages over after a
    // barrier, so the prologue is issued in two pieces.
    constexpr uint32_t STG_Q = (uint32_t)(S - 1) * 2 * P::TILE, STG_DO = (uint32_t)(S - 2) * 2 * P::TILE;
    stage_own_rows(pipe, q + own_base, I_own * BM, s.n_own, D, STG_Q);
    stage_own_rows(pipe, d_o + own_base, I_own * BM, s.n_own, D, STG_DO);
    R::start(pipe, n);
    R::template prologue<0, S - 2>(pipe, n);
    if (S == 2 || n == 0) wait_vmcnt<0>();  // otherwise the prologue's first wait covered the staged rows
    bf16x8 qf[KSTEPS], dof[KSTEPS];
#pragma unroll
    for (int st = 0; st < KSTEPS; st++) {
        qf[st] = read_row<ROWB>(smem + STG_Q, rl, wave * 32, st);
        dof[st] = read_row<ROWB>(smem + STG_DO, rl, wave * 32, st);
    }
    const int qrow_ld = min(qrow, s.n_own - 1);
    const float lse_i = lse[(size_t)bh * s.n_own + qrow_ld];
    const float2 init = row_scalars[(size_t)bh * s.n_own + qrow_ld];  // 0, 0 for a row without a key
    const float dp_init = init.x, s_init = init.y;                    // -D_i, -LSE_i / scale
    // A row without any key (a pad: LSE = -inf) is masked by the bitmap, but its Q and dO may hold anything,
    // NaN included, which a zero weight would not remove: it takes part as a row of zeros.
    const bool dead_row = lse_i == -INFINITY;
    if (dead_row) {
#pragma unroll
        for (int st = 0; st < KSTEPS; st++) qf[st] = dof[st] = zero_bf16x8();
    }
    // the compiler must finish its own loads before the hand-scheduled ones continue
    asm volatile("" ::"v"(dp_init), "v"(s_init), "v"(lse_i));
    wg_barrier();  // every wave has read its fragments: the ring may use all stages
    R::template prologue<S - 2, S - 1>(pipe, n);

    f32x16 dqacc[DBLK];
#pragma unroll
    for (int i = 0; i < DBLK; i++)
#pragma unroll
        for (int e = 0; e < 16; e++) dqacc[i][e] = 0.f;

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

#pragma unroll
        for (int kb = 0; kb < KB; kb++) {
            const int sb = wave * KB + kb;
            if (!((sub >> sb) & 1u)) continue;
            f32x16 sacc, dpacc;  // every element of a lane belongs to the lane's query
#pragma unroll
            for (int e = 0; e < 16; e++) {
                sacc[e] = s_init;
                dpacc[e] = dp_init;
            }
            // (a wave at its contractions goes before the waves of this SIMD that are at their exponentials: the
            // kernel is 3 % faster with the priorities than with the round-robin order)
            __builtin_amdgcn_s_setprio(1);
#pragma unroll
            for (int st = 0; st < KSTEPS; st++) {
                sacc = mfma_32x32x16(read_row<ROWB>(sK, rl, kb * 32, st), qf[st], sacc);     // K Q^T - LSE / scale
                dpacc = mfma_32x32x16(read_row<ROWB>(sV, rl, kb * 32, st), dof[st], dpacc);  // dP^T - D = V dO^T - D
            }
            __builtin_amdgcn_s_setprio(0);
#pragma unroll
            for (int e = 0; e < 16; e++) sacc[e] = fast_exp2(sacc[e] * scale_log2);  // P^T
            if (!((sub >> (16 + sb)) & 1u)) apply_mask(sacc, s.bits_rm + ((size_t)bidx * G::NSUB + sb) * 16, 0.f);
#pragma unroll
            for (int e = 0; e < 16; e++) sacc[e] *= dpacc[e];  // dS^T
            // dQ^T += K^T dS^T
            const bf16x8 b0 = pack_bf16x8(sacc, 0), b1 = pack_bf16x8(sacc, 8);
            __builtin_amdgcn_s_setprio(1);
#pragma unroll
            for (int j = 0; j < DBLK; j++) {
                dqacc[j] = mfma_32x32x16(read_tr<ROWB>(sK, tl, kb * 32, j), b0, dqacc[j]);
                dqacc[j] = mfma_32x32x16(read_tr<ROWB>(sK, tl, kb * 32 + 16, j), b1, dqacc[j]);
            }
            __builtin_amdgcn_s_setprio(0);
        }
    }

    {
        // through this wave's slice of the stage tile n would have used: free since the last barrier (see
        // the forward kernel), so waves leave independently
        const int wrow0 = I * BM + wave * 32;
        store_rows_via_lds<P, D>(smem + (n % S) * 2 * P::TILE + wave * 32 * ROWB, opaque(lane), dqacc, scale,
                                 dq + base + (size_t)wrow0 * D, s.n_pos - wrow0);
    }
}

// ---------------------------------------------------------------------------------------- dK, dV
// WHICH: 0 = dK and dV, 1 = dV only, 2 = dK only
template <int D, typename G, int WHICH>
__device__ __forceinline__ void dkv_role(char *smem, const HdtSchedule &s, const __bf16 *__restrict__ q,
                                          const __bf16 *__restrict__ k, const __bf16 *__restrict__ v,
                                          const __bf16 *__restrict__ d_o, const float2 *__restrict__ row_scalars,
                                          __bf16 *__restrict__ dk, __bf16 *__restrict__ dv, int wave, int I, int bh,
                                          int b, float scale)
{
    using P = Pipe<D, BwdCfg<D>::S_DKV, true, G>;
    using R = Ring<P>;
    constexpr int BM = G::BM, BN = G::BN, KB = G::KB;
    constexpr int ROWB = P::ROWB, KSTEPS = P::KSTEPS, DBLK = P::DBLK, S = P::S;
    constexpr bool DO_DV = WHICH != 2, DO_DK = WHICH != 1;

    const int lane = threadIdx.x & 63;
    const int hf = lane >> 5;
    const size_t base = (size_t)bh * s.n_pos * D, q_base = (size_t)bh * s.n_kv * D;  // rows are keys here
    const float scale_log2 = scale * LOG2E;

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
    pipe.a = q + q_base;
    pipe.b = d_o + q_base;
    pipe.aux0 = reinterpret_cast<const float *>(row_scalars + (size_t)bh * s.n_kv) + 1;  // -LSE / scale of a position
    pipe.aux1 = reinterpret_cast<const float *>(row_scalars + (size_t)bh * s.n_kv);      // -D
    const RowLane rl = row_lane<P::CPR>(lane);
    const TrLane tl = tr_lane<P::CPR>(lane);
    // is this lane's own row a real position?  (Requested first, looked at once the rows are in registers.)
    // (An unconditional load: inside a branch the compiler would wait for it on the spot.  Without flags any
    // readable word will do, its value is not used.)
    const int own_row = min(I * BM + wave * 32 + (lane & 31), s.n_pos - 1);
    const int32_t *flag_at = s.row_flag ? s.row_flag + ((size_t)b * s.n_pos + own_row) : s.q_range;
    int own_flag = *flag_at;

    // K and V rows of this wave: through the two highest ring stages, as Q and dO in the dQ pass
    constexpr uint32_t STG_K = (uint32_t)(S - 1) * 2 * P::TILE, STG_V = (uint32_t)(S - 2) * 2 * P::TILE;
    stage_own_rows(pipe, k + base, I * BM, s.n_pos, D, STG_K);
    if (DO_DK) stage_own_rows(pipe, v + base, I * BM, s.n_pos, D, STG_V);  // V only enters dP
    R::start(pipe, n);
    R::template prologue<0, S - 2>(pipe, n);
    if (S == 2 || n == 0) wait_vmcnt<0>();
    bf16x8 kf[KSTEPS], vf[KSTEPS];
#pragma unroll
    for (int st = 0; st < KSTEPS; st++) {
        kf[st] = read_row<ROWB>(smem + STG_K, rl, wave * 32, st);
        if (DO_DK) vf[st] = read_row<ROWB>(smem + STG_V, rl, wave * 32, st);
    }
    // A row that is no real position (a pad, an encoder position the decoder does not see) is masked by the
    // bitmap, but its K and V may hold anything, NaN included, which a zero weight would not remove: it takes
    // part as a row of zeros.
    if (s.row_flag != nullptr && own_flag < 0) {
#pragma unroll
        for (int st = 0; st < KSTEPS; st++) {
            kf[st] = zero_bf16x8();
            if (DO_DK) vf[st] = zero_bf16x8();
        }
    }
    wg_barrier();
    R::template prologue<S - 2, S - 1>(pipe, n);

    f32x16 dkacc[DBLK], dvacc[DBLK];
#pragma unroll
    for (int i = 0; i < DBLK; i++)
#pragma unroll
        for (int e = 0; e < 16; e++) dkacc[i][e] = dvacc[i][e] = 0.f;

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
        const char *sQ = pipe.tile_a(i % S), *sDO = pipe.tile_b(i % S);
        const float *sInitS = pipe.aux_buf(i % S, 0), *sInitDP = pipe.aux_buf(i % S, 1);  // -LSE / scale, -D

#pragma unroll
        for (int kb = 0; kb < KB; kb++) {  // 32 query slots
            const int sb = wave * KB + kb;
            if (!((sub >> sb) & 1u)) continue;
            // element gq * 4 + e of a lane belongs to the query in slot kb * 32 + hf * 4 + gq * 8 + e
            f32x16 sacc, dpacc;
#pragma unroll
            for (int gq = 0; gq < 4; gq++) {
                const float4 l4 = *reinterpret_cast<const float4 *>(&sInitS[kb * 32 + hf * 4 + gq * 8]);
                sacc[gq * 4 + 0] = l4.x;
                sacc[gq * 4 + 1] = l4.y;
                sacc[gq * 4 + 2] = l4.z;
                sacc[gq * 4 + 3] = l4.w;
                if (DO_DK) {
                    const float4 d4 = *reinterpret_cast<const float4 *>(&sInitDP[kb * 32 + hf * 4 + gq * 8]);
                    dpacc[gq * 4 + 0] = d4.x;
                    dpacc[gq * 4 + 1] = d4.y;
                    dpacc[gq * 4 + 2] = d4.z;
                    dpacc[gq * 4 + 3] = d4.w;
                }
            }
            __builtin_amdgcn_s_setprio(1);  // as in the dQ role
#pragma unroll
            for (int st = 0; st < KSTEPS; st++) {
                sacc = mfma_32x32x16(read_row<ROWB>(sQ, rl, kb * 32, st), kf[st], sacc);     // Q K^T - LSE / scale
                if (DO_DK) dpacc = mfma_32x32x16(read_row<ROWB>(sDO, rl, kb * 32, st), vf[st], dpacc);  // dO V^T - D
            }
            __builtin_amdgcn_s_setprio(0);
            f32x16 pacc;
#pragma unroll
            for (int e = 0; e < 16; e++) pacc[e] = fast_exp2(sacc[e] * scale_log2);  // P
            if (!((sub >> (16 + sb)) & 1u)) apply_mask(pacc, s.bits_rm + ((size_t)bidx * G::NSUB + sb) * 16, 0.f);
            if (DO_DK) {
#pragma unroll
                for (int e = 0; e < 16; e++) sacc[e] = pacc[e] * dpacc[e];  // dS
                const bf16x8 s0 = pack_bf16x8(sacc, 0), s1 = pack_bf16x8(sacc, 8);
                __builtin_amdgcn_s_setprio(1);
#pragma unroll
                for (int j = 0; j < DBLK; j++) {
                    dkacc[j] = mfma_32x32x16(read_tr<ROWB>(sQ, tl, kb * 32, j), s0, dkacc[j]);  // dK^T += Q^T dS
                    dkacc[j] = mfma_32x32x16(read_tr<ROWB>(sQ, tl, kb * 32 + 16, j), s1, dkacc[j]);
                }
            }
            if (DO_DV) {
                const bf16x8 p0 = pack_bf16x8(pacc, 0), p1 = pack_bf16x8(pacc, 8);
                __builtin_amdgcn_s_setprio(1);
#pragma unroll
                for (int j = 0; j < DBLK; j++) {
                    dvacc[j] = mfma_32x32x16(read_tr<ROWB>(sDO, tl, kb * 32, j), p0, dvacc[j]);  // dV^T += dO^T P
                    dvacc[j] = mfma_32x32x16(read_tr<ROWB>(sDO, tl, kb * 32 + 16, j), p1, dvacc[j]);
                }
            }
            __builtin_amdgcn_s_setprio(0);
        }
    }

    {
        // through this wave's slice of the stage tile n would have used: free since the last barrier
        const int wrow0 = I * BM + wave * 32;
        char *wl = smem + (n % S) * 2 * P::TILE + wave * 32 * ROWB;
        const int le = opaque(lane);
        if (DO_DK) store_rows_via_lds<P, D>(wl, le, dkacc, scale, dk + base + (size_t)wrow0 * D, s.n_pos - wrow0);
        if (DO_DV) store_rows_via_lds<P, D>(wl, le, dvacc, 1.f, dv + base + (size_t)wrow0 * D, s.n_pos - wrow0);
    }
}

template <int D, typename G>
__global__ __launch_bounds__(G::THREADS, BwdCfg<D>::template WAVES<G>) void k_bwd_bf16(
    HdtSchedule s, HdtSchedule s_tr, const __bf16 *__restrict__ q, const __bf16 *__restrict__ k,
    const __bf16 *__restrict__ v, const float *__restrict__ lse, const __bf16 *__restrict__ d_o,
    const float2 *__restrict__ row_scalars, __bf16 *__restrict__ dq, __bf16 *__restrict__ dk,
    __bf16 *__restrict__ dv, int heads, float scale)
{
    using PQ = Pipe<D, BwdCfg<D>::S_DQ, false, G>;
    using PK = Pipe<D, BwdCfg<D>::S_DKV, true, G>;
    constexpr int SMEM = PQ::SMEM_BYTES > PK::SMEM_BYTES ? PQ::SMEM_BYTES : PK::SMEM_BYTES;
    __shared__ __attribute__((aligned(1024))) char smem[SMEM];
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    // The roles tile different tensors (the same ones for self-attention): the workgroups of one tile follow each
    // other as far as both sides have that tile, the rest of the longer side comes behind them.
    constexpr unsigned R = BwdCfg<D>::SPLIT_KV ? 3u : 2u;  // roles per tile: dQ, then dK/dV or dV, dK
    const unsigned w = logical_block(blockIdx.x, R * G::XCD_CHUNK);
    const unsigned nq = (unsigned)s.batch * heads * s.tr, nk = (unsigned)s_tr.batch * heads * s_tr.tr;
    const unsigned common = nq < nk ? nq : nk;
    if (w >= nq + (R - 1u) * nk) return;  // padding of the grid
    unsigned role, lb;
    if (w < R * common) {
        role = w % R;
        lb = w / R;
    } else if (nq > nk) {
        role = 0u;
        lb = w - (R - 1u) * common;
    } else {
        const unsigned rest = w - R * common;
        role = 1u + rest % (R - 1u);
        lb = common + rest / (R - 1u);
    }
    if (role == 0u) {
        const int I = lb % s.tr, bh = lb / s.tr, b = bh / heads;
        dq_role<D, G>(smem, s, q, k, v, lse, d_o, row_scalars, dq, wave, I, bh, b, scale);
    } else {
        const int I = lb % s_tr.tr, bh = lb / s_tr.tr, b = bh / heads;
        if (!BwdCfg<D>::SPLIT_KV)
            dkv_role<D, G, 0>(smem, s_tr, q, k, v, d_o, row_scalars, dk, dv, wave, I, bh, b, scale);
        else if (role == 1u)
            dkv_role<D, G, 1>(smem, s_tr, q, k, v, d_o, row_scalars, dk, dv, wave, I, bh, b, scale);
        else
            dkv_role<D, G, 2>(smem, s_tr, q, k, v, d_o, row_scalars, dk, dv, wave, I, bh, b, scale);
    }
}

}  // namespace

template <typename G>
static void launch_bwd(const HdtSchedule &s, const HdtSchedule &s_tr, const __bf16 *Q, const __bf16 *K, const __bf16 *V,
                       const __bf16 *O, const float *lse, const __bf16 *DO, void *dq, void *dk, void *dv, int heads,
                       int head_dim, float scale, float *delta, hipStream_t st)
{
    // the rows' two scalars (-D, -LSE / scale), see hdt_bwd_row_scalars_bytes for the room they take
    const long long rows = (long long)s.batch * heads * s.n_own;  // the real rows, also when key lists are cut
    float2 *row_scalars = reinterpret_cast<float2 *>(delta);
    {
        HdtTimer t(head_dim == 64 ? "hdt_bwd_delta_d64" : "hdt_bwd_delta_d128", st);
        const int rpb = (256 / (head_dim / 8)) * 4;
        dim3 grid((unsigned)((rows + rpb - 1) / rpb)), block(256);
        if (head_dim == 64)
            hipLaunchKernelGGL(k_bwd_delta<64>, grid, block, 0, st, O, DO, lse, 1.f / scale, row_scalars, rows);
        else
            hipLaunchKernelGGL(k_bwd_delta<128>, grid, block, 0, st, O, DO, lse, 1.f / scale, row_scalars, rows);
    }
    {
        HdtTimer t(head_dim == 64 ? "hdt_bwd_bf16_d64" : "hdt_bwd_bf16_d128", st);
        const unsigned nq = (unsigned)s.batch * heads * s.tr, nk = (unsigned)s_tr.batch * heads * s_tr.tr;
        const unsigned roles = head_dim == 128 ? 3u : 2u;  // BwdCfg<D>::SPLIT_KV
        dim3 grid(padded_grid(nq + (roles - 1u) * nk, roles * G::XCD_CHUNK)), block(G::THREADS);
        if (head_dim == 64)
            hipLaunchKernelGGL((k_bwd_bf16<64, G>), grid, block, 0, st, s, s_tr, Q, K, V, lse, DO, row_scalars,
                               (__bf16 *)dq, (__bf16 *)dk, (__bf16 *)dv, heads, scale);
        else
            hipLaunchKernelGGL((k_bwd_bf16<128, G>), grid, block, 0, st, s, s_tr, Q, K, V, lse, DO, row_scalars,
                               (__bf16 *)dq, (__bf16 *)dk, (__bf16 *)dv, heads, scale);
    }
}

hdt_status_t hdt_launch_bwd_bf16(const HdtSchedule &s, const HdtSchedule &st_, const void *q, const void *k,
                                 const void *v, const void *o, const float *lse, const void *d_o, void *dq, void *dk,
                                 void *dv, int heads, int head_dim, float scale, float *delta, hipStream_t st)
{
    const __bf16 *Q = (const __bf16 *)q, *K = (const __bf16 *)k, *V = (const __bf16 *)v;
    const __bf16 *O = (const __bf16 *)o, *DO = (const __bf16 *)d_o;
    if (s.bm == 64)
        launch_bwd<Geo<64, 32>>(s, st_, Q, K, V, O, lse, DO, dq, dk, dv, heads, head_dim, scale, delta, st);
    else
        launch_bwd<Geo<128, 64>>(s, st_, Q, K, V, O, lse, DO, dq, dk, dv, heads, head_dim, scale, delta, st);
    HDT_HIP_TRY(hipGetLastError());
    return HDT_OK;
}
