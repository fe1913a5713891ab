// Tile movement and fragment helpers shared by the tuned bf16 attention kernels (block size 32 or 64).
//   - tiles travel HBM -> LDS through the memory pipeline (global_load_lds): no staging registers,
//     no LDS stores;
//   - tiles stay row-major in LDS, 16-byte slots permuted per row so that no read conflicts;
//     operands that must be read along the row index come out of the same tile through the LDS
//     transpose read (ds_read_b64_tr_b16: 16 lanes fetch a 4 x 16 patch, each receives a column).
#ifndef SPION_ATTN_BF16_TILES_H_
#define SPION_ATTN_BF16_TILES_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "attn_common.h"

namespace spion {

__device__ __forceinline__ bf16x4 lds_read_tr(const bf16_t* p) {
    typedef bf16x4 __attribute__((address_space(3))) * lds_ptr;
    return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_ptr)p);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Workgroups are dealt round-robin to the 8 XCDs in id order.  Give XCD x the x-th contiguous
// eighth of the (head-major) work so that the K / V (or Q / dO) rows of a head stay in one L2.
__device__ __forceinline__ int xcd_remap(int id, int total) {
    if (total & 7) return id;
    return (id & 7) * (total >> 3) + (id >> 3);
}

// ------------------------------------------------------------------------------------------------
// Tiles loaded by the memory pipeline straight into LDS (global_load_lds, 16 B per lane; a wave
// instruction fills 1 KB of consecutive LDS, lane l at byte 16 l).  Rows are 128 B apart with no
// padding, so the 16-byte slots of a row are permuted instead: slot s of row `row` holds the row's
// chunk s ^ swz(row), swz = 2 * ((row >> 1) & 3).  Measured with SQ_LDS_BANK_CONFLICT: neither the
// 16-byte fragment reads (lane = row) nor the transpose reads (8 rows x 32 B per half wave) conflict
// in this layout.  (A 16-byte read is served 16 lanes at a time, lanes 0-7 together with lanes of the
// upper half of a neighbouring group of 16: a permutation that also used bit 3 of the row conflicted.)
// ------------------------------------------------------------------------------------------------
typedef __attribute__((address_space(3))) void* lds_void_ptr;

// s_waitcnt immediates (gfx9 encoding: vmcnt [3:0] and [15:14], expcnt [6:4], lgkmcnt [11:8]); the
// counters not named are left at their maximum, i.e. not waited for
constexpr int kWaitVm0 = 0x0F70, kWaitVm4 = 0x0F74, kWaitVm5 = 0x0F75, kWaitLgkm0 = 0xC07F;

__device__ __forceinline__ int swz(int row) { return ((row >> 1) & 3) << 1; }

// A workgroup of BS / 16 waves loads a BS x 64 tile with two instructions per wave.  `src` and
// `wave` are wave-uniform (the wave index comes from readfirstlane), so each load is a scalar base
// plus the lane's fixed 32-bit offset TileLoadLane::off[k].
struct TileLoadLane {
    unsigned off[2];   // byte offset of this lane's 16 bytes within the tile, for piece 2 wave + k
    __device__ __forceinline__ TileLoadLane(int wave, int lane) {
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const int chunk = (lane & 7) ^ (((lane >> 4) & 3) << 1);   // swz(8 piece + lane / 8)
            off[k] = (unsigned)(((2 * wave + k) * 8 + (lane >> 3)) * kD + chunk * 8) * (unsigned)sizeof(bf16_t);
        }
    }
};
__device__ __forceinline__ void tile_load_async(const bf16_t* __restrict__ src, bf16_t* tile, int wave,
                                                const TileLoadLane& tl) {
#pragma unroll
    for (int k = 0; k < 2; ++k)
        __builtin_amdgcn_global_load_lds(reinterpret_cast<const char*>(src) + tl.off[k],
                                         (lds_void_ptr)(tile + (2 * wave + k) * 512), 16, 0, 0);
}

// Per-lane read offsets into such a tile (in elements), fixed for the whole kernel.
struct SwzLane {
    int frag[2];   // 16-byte fragment of row r, chunk 4 c + g; add 1024 per 16-row tile
    int tr_row;    // transpose read: row 4 g + r / 4, element offset 4 (r & 1) within the slot
    int tr_sw;     // swz of that row
    int tr_b;      // (r >> 1) & 1: which slot of the 32-byte pair
    __device__ __forceinline__ SwzLane(int r, int g) {
        const int sw = swz(r);
        frag[0] = r * kD + ((g ^ sw) << 3);
        frag[1] = r * kD + (((4 + g) ^ sw) << 3);
        const int trow = 4 * g + (r >> 2);
        tr_row = trow * kD + 4 * (r & 1);
        tr_sw = swz(trow);
        tr_b = (r >> 1) & 1;
    }
    __device__ __forceinline__ int tr(int dt) const { return tr_row + ((((dt << 1) | tr_b) ^ tr_sw) << 3); }
};

// acc[dt][i] (d = 16 dt + 4 g + i, owned row r) += sum over the tile's rows of
// tile[row][16 dt + ...] * x[row][r], the tile in the permuted-slot layout.
template <int BS>
__device__ __forceinline__ void mma_over_rows_swz(f32x4 (&acc)[4], const bf16_t* tile,
                                                  const bf16x4 (&x)[BS / 16], const SwzLane& sl) {
#pragma unroll
    for (int pc = 0; pc < BS / 32; ++pc) {
        const bf16x8 xf = join(x[2 * pc], x[2 * pc + 1]);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
            const int o = sl.tr(dt) + pc * 32 * kD;
            acc[dt] = mma_d(acc[dt], join(lds_read_tr(tile + o), lds_read_tr(tile + 16 * kD + o)), xf);
        }
    }
}

// Write this wave's 16 owned rows x 64 columns (accumulators in the transposed layout: lane (r, g)
// holds columns 16 dt + 4 g .. + 3 of row r) as whole 128-byte rows, 16 bytes per lane, instead of
// 8-byte pieces: through a 2 KB LDS patch private to the wave, 16-byte chunks permuted by the row.
// LDS instructions of one wave execute in order, so no barrier is needed between the two halves.
__device__ __forceinline__ void store_rows_coalesced(bf16_t* patch, bf16_t* __restrict__ grow0,
                                                     const f32x4 (&acc)[4], float mul, int lane) {
    const int r = lane & 15, g = lane >> 4;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
        const int chunk = (dt * 2 + (g >> 1)) ^ (r & 7);
        *reinterpret_cast<bf16x4*>(patch + r * kD + chunk * 8 + (g & 1) * 4) = to_quad<bf16_t>(acc[dt] * mul);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int row = (lane >> 3) + 8 * j, c = lane & 7;
        const bf16x8 v = *reinterpret_cast<const bf16x8*>(patch + row * kD + ((c ^ (row & 7)) << 3));
        *reinterpret_cast<bf16x8*>(grow0 + (size_t)row * kD + c * 8) = v;
    }
}

// Walk order of a block row.  The diagonal block (I, I) is kept by every pattern the generator makes,
// and its address needs no index lookup, so the row-walking kernels start loading it before they
// have read row_ptr / col_idx and visit it first; the other kept blocks follow in index order.  (The
// order of the blocks changes the rounding of the sums only.)  pd = position of I among the row's
// entries, or -1 if the row has no diagonal block: then the walk is in index order and the early
// load is thrown away.
// Scalar loads on purpose: they do not count against the vector-memory counter, so waiting for
// them does not wait for the tile loads already in flight.  The entries of a row ascend, so the scan
// stops at the first entry >= I.  first[] receives entries 0..7 (clamped to the row), from which
// the first blocks of the walk are taken without another dependent load.
__device__ __forceinline__ int find_in_row(const int* __restrict__ cols, int n, int I, int (&first)[8]) {
    const int last = n - 1;
    int pd = -2;   // -2: not decided yet
#pragma unroll
    for (int e = 0; e < 8; ++e) first[e] = cols[e < last ? e : last];
#pragma unroll
    for (int e = 0; e < 8; ++e)
        if (pd == -2 && first[e] >= I) pd = (first[e] == I && e < n) ? e : -1;
    for (int base = 8; base < n && pd == -2; base += 8) {
        int c[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) c[e] = cols[base + e < last ? base + e : last];
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (pd == -2 && c[e] >= I) pd = (c[e] == I && base + e < n) ? base + e : -1;
    }
    return pd == -2 ? -1 : pd;
}
__device__ __forceinline__ int pick8(const int (&v)[8], int i) {
    const int a = (i & 1) ? v[1] : v[0], b = (i & 1) ? v[3] : v[2], c = (i & 1) ? v[5] : v[4],
              d = (i & 1) ? v[7] : v[6];
    const int ab = (i & 2) ? b : a, cd = (i & 2) ? d : c;
    return (i & 4) ? cd : ab;
}
__device__ __forceinline__ int walk_index(int t, int pd) {
    return pd < 0 ? t : (t == 0 ? pd : (t - 1 < pd ? t - 1 : t));
}

}  // namespace spion
#endif
