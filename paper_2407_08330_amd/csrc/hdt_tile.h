// Pieces shared by the three bf16 kernels (forward, dQ pass, dK/dV pass).  All of them have the same
// skeleton: a workgroup of BM/32 waves owns BM consecutive rows of the schedule (wave w the rows
// 32w..32w+31, whose operands stay in registers as MFMA B fragments), walks the row tile's list
// entries, and for each entry gathers the BN rows of two [n_pos][D] tensors that the entry's key
// positions name into LDS.  Two tile shapes are built: 128 x 64 (four waves; the layout's default) and
// 64 x 32 (two waves).  The waves of a workgroup meet at a barrier once per entry and the mask is close to
// block diagonal, so with four waves a wave often waits through entries that hold nothing for its rows;
// the finer shape loses fewer such slots and skips more of the mask, but walks more entries and needs
// twice the workgroups.  Measured, the two are within a few percent of each other at head size 64 and the
// finer one is ~5-10 % ahead at head size 128, before the doubled cost of building its layout.
//
// The gather uses the CDNA direct-to-LDS loads (global_load_lds_*: every lane supplies a global
// address, the 64 results land in LDS at M0 + lane*size) into a ring of S stages, so that several
// tiles are in flight per workgroup without holding them in registers:
//   iteration t:  wait until tile t has landed -> barrier -> start tile t+S-1 -> compute tile t.
// The key positions of an entry are read the same way, one tile further ahead than the rows they
// address, and the entries' summaries with scalar loads, so no iteration waits on a chain of dependent
// loads.
// The only vector-memory instructions inside the loop are those issued here with inline asm, which
// is what makes the hand-counted s_waitcnt vmcnt(N) exact.
//
// A wave-level load writes 1024 contiguous bytes, so LDS rows cannot be padded; bank conflicts are
// avoided with an XOR swizzle of the 16-byte chunks of a row instead (applied to the global address
// of each lane on the way in, and to the LDS address on the way out).
#pragma once

#include "hdt_internal.h"
#include "hdt_mfma.h"

namespace hdt_tile {

// tile geometry: BM query rows x BN key slots, one wave per 32 rows; a ring stage (two tiles of BN rows)
// also has to hold the workgroup's own BM rows, hence BM = 2 BN, and every wave loads 16 rows of a tile
template <int BM_, int BN_>
struct Geo {
    static constexpr int BM = BM_, BN = BN_;
    static constexpr int NW = BM_ / 32;               // waves per workgroup
    static constexpr int THREADS = NW * 64;
    static constexpr int KB = BN_ / 32;               // 32-key sub-blocks per tile
    static constexpr int NSUB = (BM_ / 32) * KB;      // 32x32 sub-blocks per tile
    static constexpr unsigned XCD_CHUNK = 4096 / BM_; // consecutive row tiles handed to one XCD (see logical_block)
    static_assert(BM_ == 2 * BN_ && BN_ / NW == 16, "unsupported tile shape");
};
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

// Read-only schedule arrays are read through the constant address space: with a wave-uniform index
// the compiler then uses scalar loads (lgkmcnt), which keeps them out of the vector-memory queue
// whose in-order counter the hand-scheduled loads rely on.
#define HDT_CONST __attribute__((address_space(4)))
typedef const int32_t HDT_CONST *cptr_i32;
typedef const uint32_t HDT_CONST *cptr_u32;
__device__ __forceinline__ cptr_i32 as_const(const int32_t *p) { return (cptr_i32)(uintptr_t)p; }
__device__ __forceinline__ cptr_u32 as_const(const uint32_t *p) { return (cptr_u32)(uintptr_t)p; }

// Workgroups are handed to the 8 XCDs round-robin (workgroup id mod 8).  Logical work items are dealt to
// the XCDs in chunks of consecutive items (Geo::XCD_CHUNK row tiles: 4096 rows), so that neighbouring row tiles
// (which gather largely the same rows) share an L2, while every XCD still gets an even mix of the samples: with
// whole (sample, head) ranges per XCD, one long document made two XCDs finish well after the others.  The chunk
// is counted in rows: with 32 tiles of 64 rows the forward took 48.8 us at 8192 positions x 4 samples x 12
// heads, with 64 of them 46.4, as with 32 tiles of 128 rows.  Every round of 8 chunks starts one XCD further: a
// sample of 8192 positions is two chunks, and the first halves of documents that end in pads are the heavier
// ones, which would otherwise all go to the even XCDs (7 % more work there).  The grid is padded to a multiple
// of 8 chunks; padding workgroups get an index >= n_items and leave at once.
__host__ __device__ __forceinline__ unsigned padded_grid(unsigned n_items, unsigned chunk)
{
    return (n_items + 8u * chunk - 1u) / (8u * chunk) * (8u * chunk);
}
__device__ __forceinline__ unsigned logical_block(unsigned bid, unsigned chunk)
{
    const unsigned x = bid & 7u, k = bid >> 3, round = k / chunk;
    return (round * 8u + ((x + round) & 7u)) * chunk + k % chunk;
}

// Chunk swizzle of row r of a tile whose rows hold CPR chunks of 16 bytes.  The LDS has 64 banks of 4 bytes
// (256 bytes per clock): a 16-byte read is served 16 lanes at a time, a transposing 8-byte read 32 lanes at
// a time, and a group is conflict-free when its lanes fall into different 16-byte columns of the 256.
//   row reads (one logical chunk down 16 consecutive rows): 16 different columns.  With 128-byte rows the
//     row's parity picks the half of the 256 bytes, so the 8 even rows need 8 different values and so do the
//     8 odd ones; with 256-byte rows all 16 values differ.
//   transposing reads (4 consecutive aligned rows x 4 chunks 4i ^ {0..3}): the rows that share a half must
//     differ in the chunk bits above the low two.
// Rows r and r + 8 differ by 2 in both cases (what the second of a pair of transposing reads relies on).
// Measured on the chip: 4.0 clocks per 16-byte wave read against 6.4 with a swizzle of period 8.
template <int CPR>
__device__ __forceinline__ int swz(int r)
{
    if (CPR == 8) return (((r & 3) << 1) | ((r >> 2) & 1)) ^ ((r >> 2) & 2);
    return ((r & 3) << 2) | ((r >> 2) & 3);
}

__device__ __forceinline__ uint32_t lds_addr(const void *p)
{
    return (uint32_t)(uintptr_t)(HDT_LDS const char *)p;
}

// direct-to-LDS loads: lane l's 16 (4) bytes at base + off (a wave-uniform base pointer in scalar registers,
// a per-lane byte offset below 2^31) land at lds_base + 16*l (4*l)
__device__ __forceinline__ void dma16(const void *base, uint32_t off, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(base), "s"(lds_base)
                 : "memory", "m0");
}
__device__ __forceinline__ void dma4(const void *base, uint32_t off, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" ::"v"(off), "s"(base), "s"(lds_base)
                 : "memory", "m0");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// workgroup barrier without the fence __syncthreads() carries: LDS traffic of this wave is drained
// by the lgkmcnt wait, the direct-to-LDS loads by the explicit vmcnt waits of the callers
__device__ __forceinline__ void wg_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// The row to gather for a key slot.  A slot without a key holds ~f, f being a position of the same sample that
// some row of the tile may attend to: its rows are finite whenever the tile's real rows are, so the zero weights
// the bitmap gives the slot never meet a non-finite operand (pad rows may hold anything).
__device__ __forceinline__ int gather_row(int slot_value) { return slot_value ^ (slot_value >> 31); }

template <int D, int S_, bool AUX, typename G>
struct Pipe {
    static constexpr int BM = G::BM, BN = G::BN, NW = G::NW;
    static constexpr int S = S_;                      // data stages in the ring
    static constexpr int PS = 4;                      // position stages
    static constexpr int KSTEPS = D / 16;             // MFMA steps over the head dimension
    static constexpr int DBLK = D / 32;               // 32-wide blocks of the head dimension
    static constexpr int ROWB = D * 2;                // bytes per LDS row (unpadded)
    static constexpr int CPR = D / 8;                 // 16-byte chunks per row
    static constexpr int TILE = BN * ROWB;            // bytes of one gathered tile of one tensor
    static constexpr int RPI = 1024 / ROWB;           // rows per wave-level load
    static constexpr int LPW = BN / NW;               // rows of a tile each wave loads (16)
    static constexpr int NI = LPW / RPI;              // wave-level loads per tensor per tile per wave
    static constexpr int POSW = 64;                   // ints per position buffer (one wave-level load; BN are used)
    static constexpr int NDMA = 2 * NI + (AUX ? 1 : 0);  // vector-memory instructions per tile per wave
    static constexpr int DATA_BYTES = S * 2 * TILE;
    static constexpr int POS_BYTES = PS * NW * POSW * 4;
    static constexpr int AUX_BYTES = AUX ? S * NW * POSW * 4 : 0;
    static constexpr int SMEM_BYTES = DATA_BYTES + POS_BYTES + AUX_BYTES;

    char *smem;
    uint32_t smem_addr;
    int wave, lane;
    const int32_t *keys;       // key positions of this row tile's entries: [n][BN]
    const __bf16 *a, *b;       // the two gathered tensors, already offset to this (sample, head)
    const float *aux0, *aux1;  // per-position floats gathered with the rows (AUX only): the two halves of an array
                               // of float pairs, hence 8 bytes from one position to the next

    __device__ __forceinline__ const char *tile_a(int stage) const { return smem + (stage * 2 + 0) * TILE; }
    __device__ __forceinline__ const char *tile_b(int stage) const { return smem + (stage * 2 + 1) * TILE; }
    __device__ __forceinline__ const int *pos_buf(int ps) const
    {
        return reinterpret_cast<const int *>(smem + DATA_BYTES) + (ps * NW + wave) * POSW;
    }
    // aux values of the 64 slots: array 0 is written by wave 0, array 1 by wave 1
    __device__ __forceinline__ const float *aux_buf(int stage, int which) const
    {
        return reinterpret_cast<const float *>(smem + DATA_BYTES + POS_BYTES) + (stage * NW + which) * POSW;
    }

    // start loading the key positions of the row tile's j-th entry (every wave keeps its own copy)
    __device__ __forceinline__ void issue_pos(int j, int ps) const
    {
        // (64 lanes load; with BN = 32 the upper half repeats the lower one)
        dma4(keys + j * BN, (uint32_t)(lane & (BN - 1)) * 4u, smem_addr + DATA_BYTES + ((ps * NW + wave) * POSW) * 4);
    }

    // start gathering the rows of an entry whose positions sit in position stage ps
    __device__ __forceinline__ void issue_data(int stage, int ps) const
    {
        const int *pb = pos_buf(ps);
        const int lr = lane / CPR, c = lane % CPR;  // row inside the wave-level load, chunk slot
#pragma unroll
        for (int i = 0; i < NI; i++) {
            const int r = wave * LPW + i * RPI + lr;
            const int pos = gather_row(pb[r]);
            const uint32_t off = (uint32_t)pos * ROWB + (uint32_t)((c ^ swz<CPR>(r)) * 16);  // bytes
            const uint32_t dst = (uint32_t)((wave * LPW + i * RPI) * ROWB);
            dma16(a, off, smem_addr + (stage * 2 + 0) * TILE + dst);
            dma16(b, off, smem_addr + (stage * 2 + 1) * TILE + dst);
        }
        if (AUX) {
            const int pos = gather_row(pb[lane & (BN - 1)]);
            const float *src = (wave & 1) ? aux1 : aux0;
            dma4(src, (uint32_t)pos * 8u, smem_addr + DATA_BYTES + POS_BYTES + ((stage * NW + wave) * POSW) * 4);
        }
    }
};

// vmcnt wait with a run-time count out of a small set (the immediate must be a constant)
// k tiles were started after the one waited for: k*NDMA row loads and k-1 position loads
template <int NDMA>
__device__ __forceinline__ void wait_vmcnt_tail(int k)
{
    if (k <= 0)
        wait_vmcnt<0>();
    else if (k == 1)
        wait_vmcnt<NDMA>();
    else if (k == 2)
        wait_vmcnt<2 * NDMA + 1>();
    else
        wait_vmcnt<3 * NDMA + 2>();  // also safe (stricter) for k > 3
}

// Ring schedule (positions run one tile ahead of their rows).  Per wave the vector-memory
// instructions are issued in the order  pos(0), pos(1), data(0), pos(2), data(1), ..., pos(j+1), data(j), ...
// where data(j) is NDMA instructions and pos(j) one.
//   start(n), prologue(n): start pos(0..S-1) and data(0..S-2) as far as they exist
//   top(i, n):         call at the top of iteration i: returns when data(i) and pos(i+S-1) have landed
//                      in LDS for this wave; the caller then executes a workgroup barrier
//   advance(i, n):     after the barrier: starts pos(i+S) and data(i+S-1)
template <typename P>
struct Ring {
    static constexpr int S = P::S, NDMA = P::NDMA, PS = P::PS;

    // first half of the prologue: pos(0), pos(1).  The caller may issue its own (compiler-scheduled)
    // loads after this and before prologue(); the compiler's wait for those also covers these two.
    static __device__ __forceinline__ void start(const P &p, int n)
    {
        if (n > 0) p.issue_pos(0, 0);
        if (n > 1) p.issue_pos(1, 1);
    }

    // second half: pos(j+1), data(j) for j in [J0, J1) (the whole prologue is J0 = 0, J1 = S-1; it may be
    // issued in two pieces when some ring stages are still in use, see the backward kernels)
    template <int J0, int J1>
    static __device__ __forceinline__ void prologue(const P &p, int n)
    {
#pragma unroll
        for (int j = J0; j < J1; j++) {
            if (j > 0 && j + 1 < n) p.issue_pos(j + 1, (j + 1) % PS);
            if (j < n) {
                // pos(j) must have landed; issued after it: [data(j-1)], [pos(j+1)]
                if (j == 0) {
                    if (1 < n) wait_vmcnt<1>(); else wait_vmcnt<0>();
                } else {
                    if (j + 1 < n) wait_vmcnt<NDMA + 1>(); else wait_vmcnt<NDMA>();
                }
                p.issue_data(j % S, j % PS);
            }
        }
    }

    static __device__ __forceinline__ void top(int i, int n)
    {
        if (i + S - 1 < n) {
            // the last instructions issued were pos(i+S-1), data(i+S-2): with S >= 3 the latter may stay
            // in flight, with S == 2 it is data(i) itself
            wait_vmcnt<(S >= 3) ? NDMA : 0>();
        } else {
            // nothing more to start: data(i+1 .. n-1) and the position loads between them may be in flight
            wait_vmcnt_tail<NDMA>(n - 1 - i);
        }
    }

    static __device__ __forceinline__ void advance(const P &p, int i, int n)
    {
        if (i + S < n) p.issue_pos(i + S, (i + S) % PS);
        if (i + S - 1 < n) p.issue_data((i + S - 1) % S, (i + S - 1) % PS);
    }
};

// A wave's own 32 rows of a [n_pos][D] tensor (rows row0 + 32*wave .. +31, clamped to n_pos-1),
// loaded straight into LDS as rows 32*wave .. of a swizzled tile at byte offset lds_off: full rows per
// 8 or 16 lanes, so every 128-byte line is fetched once.  The MFMA B fragments of those rows are
// then read back with read_row().  Issues 32/RPI vector-memory instructions.
template <typename P>
__device__ __forceinline__ void stage_own_rows(const P &p, const __bf16 *t, int row0, int n_pos, int D, uint32_t lds_off)
{
    const int lr = p.lane / P::CPR, c = p.lane % P::CPR;
#pragma unroll
    for (int i = 0; i < 32 / P::RPI; i++) {
        const int r = p.wave * 32 + i * P::RPI + lr;
        const int g = min(row0 + r, n_pos - 1);
        dma16(t, (uint32_t)g * P::ROWB + (uint32_t)((c ^ swz<P::CPR>(r)) * 16),
              p.smem_addr + lds_off + (uint32_t)((p.wave * 32 + i * P::RPI) * P::ROWB));
    }
}

// A value the compiler cannot see through: what is derived from it is computed after this point.  Used on
// the lane index in front of an epilogue, whose per-lane addresses would otherwise be hoisted above the
// tile loop and held in registers throughout it.
__device__ __forceinline__ int opaque(int x)
{
    asm volatile("" : "+v"(x));
    return x;
}

// Epilogue: a wave's 32 x D accumulator block, held transposed in C fragments (lane (row l%32, hf)
// holds columns 32j + 4hf + 8g + 0..3), is scaled, rounded to bf16, transposed through a wave-private
// LDS area of 32*ROWB bytes and written to global memory as full rows (16 bytes per lane).
template <typename P, int D>
__device__ __forceinline__ void store_rows_via_lds(char *wave_lds, int lane, const f32x16 (&acc)[D / 32], float mult,
                                                   __bf16 *dst, int rows_valid)
{
    const int r = lane & 31, hf = lane >> 5;
#pragma unroll
    for (int j = 0; j < D / 32; j++)
#pragma unroll
        for (int gq = 0; gq < 4; gq++) {
            bf16x4 w;
#pragma unroll
            for (int e = 0; e < 4; e++) w[e] = (__bf16)(acc[j][gq * 4 + e] * mult);
            const int cl = j * 4 + gq;  // 16-byte chunk holding columns 32j + 8gq .. +7
            *reinterpret_cast<bf16x4 *>(wave_lds + r * P::ROWB + ((cl ^ (r & 7)) << 4) + hf * 8) = w;
        }
    const int lr = lane / P::CPR, c = lane % P::CPR;
#pragma unroll
    for (int i = 0; i < 32 / P::RPI; i++) {
        const int row = i * P::RPI + lr;
        const u32x4 v = *reinterpret_cast<const u32x4 *>(wave_lds + row * P::ROWB + ((c ^ (row & 7)) << 4));
        // streaming store: results are not read again by this launch and should not displace its inputs in L2
        if (row < rows_valid) __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(dst + (size_t)row * D + c * 8));
    }
}

// Per-lane constants for reading MFMA A operands by rows out of a swizzled tile: the lane's row
// inside a 32-row block and its swizzle term; 16-byte chunk 2*st + hf of that row sits at
// ((2*st) ^ x) * 16.
struct RowLane {
    int row;  // l % 32
    int x;    // hf ^ swz(row)
};
template <int CPR>
__device__ __forceinline__ RowLane row_lane(int lane)
{
    RowLane r;
    r.row = lane & 31;
    r.x = (lane >> 5) ^ swz<CPR>(r.row);
    return r;
}
template <int ROWB>
__device__ __forceinline__ bf16x8 read_row(const char *tile, const RowLane &r, int r0, int st)
{
    return lds_read_8(tile + (r0 + r.row) * ROWB + ((((st << 1) ^ r.x)) << 4));
}

// Per-lane constants of the transposing reads of a 32(k) x 32(n) operand block out of a swizzled
// row-major tile: row of the first read and the swizzle term; the chunk of n-block i is (4i) ^ y.
struct TrLane {
    int row;   // (g>>1)*4 + (tl>>2)
    int y;     // ((g&1)*2 + ((tl&3)>>1)) ^ swz(row)
    int half;  // (tl & 1) * 8 bytes inside the chunk
};
template <int CPR>
__device__ __forceinline__ TrLane tr_lane(int lane)
{
    const int g = lane >> 4, tl = lane & 15;
    TrLane t;
    t.row = (g >> 1) * 4 + (tl >> 2);
    t.y = (((g & 1) << 1) | ((tl & 3) >> 1)) ^ swz<CPR>(t.row);
    t.half = (tl & 1) * 8;
    return t;
}
// the 8 contraction values {k0 + hf*4 + 0..3} and {k0 + 8 + hf*4 + 0..3} at n = 32*i + l%32 (k0 a multiple of 16:
// the rows of the second read sit 8 further down, where the swizzle differs by 2)
template <int ROWB>
__device__ __forceinline__ bf16x8 read_tr(const char *tile, const TrLane &t, int k0, int i)
{
    const char *p0 = tile + (k0 + t.row) * ROWB + ((((i << 2) ^ t.y)) << 4) + t.half;
    const char *p1 = tile + (k0 + 8 + t.row) * ROWB + ((((i << 2) ^ t.y ^ 2)) << 4) + t.half;
    return lds_read_tr_8(p0, p1);
}

// Apply a 32x32 sub-block's bitmap to a C fragment: element e of lane l is kept iff bit l of
// mask[e] is set (the "register-major" bitmap the layout stores per sub-block), else replaced.
// The 16 masks are fetched with scalar loads (the address is the same for the whole wave; the
// layout is read-only while attention kernels run) and used directly as the lane masks of
// v_cndmask (a wave-uniform 64-bit value turned into a per-lane condition).
typedef const unsigned long long __attribute__((address_space(4))) hdt_cmask_t;

__device__ __forceinline__ void apply_mask(f32x16 &x, const unsigned long long *mask, float fill)
{
    hdt_cmask_t *cm = (hdt_cmask_t *)(uintptr_t)mask;
#pragma unroll
    for (int e = 0; e < 16; e++) x[e] = __builtin_amdgcn_inverse_ballot_w64(cm[e]) ? x[e] : fill;
}

}  // namespace hdt_tile
