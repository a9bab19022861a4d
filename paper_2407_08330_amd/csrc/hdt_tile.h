// Pieces shared by the three bf16 kernels (forward, dQ pass, dK/dV pass).  All of them have the same
// skeleton: a workgroup of 4 waves owns 128 consecutive rows of the schedule (wave w the rows
// 32w..32w+31, whose operands stay in registers as MFMA B fragments), walks the row tile's list of
// column tiles, and for each column tile gathers 64 rows of two [n_pos][D] tensors through kperm into
// LDS.  Global loads run one tile ahead of the compute, the kperm look-ups two tiles ahead and the
// list entries three tiles ahead, so that no iteration waits on a chain of dependent loads.
#pragma once

#include "hdt_internal.h"
#include "hdt_mfma.h"

namespace hdt_tile {

constexpr int BM = 128, BN = 64, THREADS = 256;
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

// One list entry: column tile, 32x32 sub-block summary, index of its bitmaps.
struct Entry {
    int col;
    uint32_t sub;
    int bidx;
};

__device__ __forceinline__ Entry load_entry(const HdtSchedule &s, int t, int t_end)
{
    Entry e{0, 0u, 0};
    if (t < t_end) {
        e.col = s.q_cols[t];
        e.sub = s.q_sub[t];
        e.bidx = s.q_bidx[t];
    }
    return e;
}

// Workgroups are handed to the 8 XCDs round-robin; give each XCD a contiguous range of logical
// work items so that the row tiles of one (sample, head) share an L2.
__device__ __forceinline__ unsigned logical_block(unsigned bid, unsigned grid)
{
    if (grid % 8u) return bid;
    return (bid % 8u) * (grid / 8u) + bid / 8u;
}

template <int D>
struct Geom {
    static constexpr int KSTEPS = D / 16;              // MFMA steps over the head dimension
    static constexpr int DBLK = D / 32;                // 32-wide blocks of the head dimension
    static constexpr int CPR = D / 8;                  // 16-byte chunks per row
    static constexpr int NLD = BN * CPR / THREADS;     // chunks per thread per gathered tile
    static constexpr int RPP = THREADS / CPR;          // rows covered by one load pass
    static constexpr int ROW_STRIDE = D * 2 + 16;      // LDS row stride for tiles read by rows
    static constexpr int TR_STRIDE = D * 2 + 32;       // ... for tiles (also) read transposed
};

// gather positions of column tile `col` for this thread's rows
template <int D>
__device__ __forceinline__ void load_positions(const int32_t *kperm, int col, int ld_row, int (&pos)[Geom<D>::NLD])
{
#pragma unroll
    for (int p = 0; p < Geom<D>::NLD; p++) {
        const int v = kperm[col * BN + ld_row + p * Geom<D>::RPP];
        pos[p] = v < 0 ? 0 : v;  // slots past n_pos: any readable row, the bitmap masks them
    }
}

template <int D>
__device__ __forceinline__ void gather_rows(const __bf16 *__restrict__ a, const __bf16 *__restrict__ b, size_t base,
                                            const int (&pos)[Geom<D>::NLD], int ld_ch, u32x4 (&ra)[Geom<D>::NLD],
                                            u32x4 (&rb)[Geom<D>::NLD])
{
#pragma unroll
    for (int p = 0; p < Geom<D>::NLD; p++) {
        const size_t off = base + (size_t)pos[p] * D + ld_ch * 8;
        ra[p] = *reinterpret_cast<const u32x4 *>(a + off);
        rb[p] = *reinterpret_cast<const u32x4 *>(b + off);
    }
}

template <int D, int STRIDE_A, int STRIDE_B>
__device__ __forceinline__ void stage_rows(char *sa, char *sb, int ld_row, int ld_ch,
                                           const u32x4 (&ra)[Geom<D>::NLD], const u32x4 (&rb)[Geom<D>::NLD])
{
#pragma unroll
    for (int p = 0; p < Geom<D>::NLD; p++) {
        const int r = ld_row + p * Geom<D>::RPP;
        *reinterpret_cast<u32x4 *>(sa + r * STRIDE_A + ld_ch * 16) = ra[p];
        *reinterpret_cast<u32x4 *>(sb + r * STRIDE_B + ld_ch * 16) = rb[p];
    }
}

// Apply a 32x32 sub-block's bitmap to a C fragment: element e of lane l is kept iff bit l of
// mask[e] is set (the "register-major" bitmap the layout stores per sub-block), else replaced.
// The 16 masks are fetched with scalar loads (the address is the same for the whole wave; the
// layout is read-only while attention kernels run) and used directly as v_cndmask lane masks.
typedef const unsigned long long __attribute__((address_space(4))) hdt_cmask_t;

__device__ __forceinline__ void apply_mask(f32x16 &x, const unsigned long long *mask, float fill)
{
    hdt_cmask_t *cm = (hdt_cmask_t *)(uintptr_t)mask;
#pragma unroll
    for (int e = 0; e < 16; e++) {
        const unsigned long long m = cm[e];
        float r;
        asm volatile("v_cndmask_b32_e64 %0, %1, %2, %3" : "=v"(r) : "v"(fill), "v"(x[e]), "s"(m));
        x[e] = r;
    }
}

// byte offset, inside a row-major LDS tile with the given row stride, of this lane's first
// transposing read for the 32(k) x 32(n) operand block whose first k-row is k0 and first n is n0
__device__ __forceinline__ int tr_offset(int lane, int stride)
{
    const int g = lane >> 4, tl = lane & 15;
    return ((g >> 1) * 4 + (tl >> 2)) * stride + ((g & 1) * 16 + (tl & 3) * 4) * 2;
}

}  // namespace hdt_tile
