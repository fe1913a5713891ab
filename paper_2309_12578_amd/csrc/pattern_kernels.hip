// Pattern generation kernels for gfx950 (Algorithm 3 and Algorithm 4 of the SPION paper).
//
//   conv_pool_kernel      Eq. 3 + Eq. 4 fused: one streaming pass over A^s that splits every input
//                         block's (fixed-point) scores over the <= 7 pooled blocks its diagonal filter
//                         window touches and writes each of the seven sums into a slot of the record
//                         of the pooled block it belongs to.  HBM bound: A^s is read exactly once,
//                         nothing L x L is written, no atomics.
//   pattern_finish_kernel one workgroup: adds the records up into pool_sum, then threshold (exact
//                         order statistic / mean + k std),
//                         successor bits, anti-diagonal wavefront flood fill, forced diagonal,
//                         BSR + BSC compaction.  Latency bound (nb^2 <= ~1M cells).
//
// Arithmetic: a_q = rint(a * 2^40) as an exact integer; all sums are integer, so any summation
// order (tiling, partial records) gives the same bits.  This file is compiled with -ffp-contract=off: the
// fp64 mean / std threshold must round exactly as its sequential definition.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "spion_internal.h"

namespace spion {

// ------------------------------------------------------------------------------------------------
// conv + pool
// ------------------------------------------------------------------------------------------------
// Input block (I, J) of A^s (bs x bs scores).  conv_out(i, j) = sum_{g=-p..p} a(i+g, j+g), so the
// score at local position (u, v) of this block is added to the outputs (u-g, v-g), g in [-p, p].
// Those outputs fall into blocks (I+di, J+dj) with di, dj in {-1, 0, +1} (p < bs) and never into
// (-1,+1) or (+1,-1) because g shifts both coordinates alike.  The number of g landing in
// (di, dj) is the size of an interval intersection, a small integer weight w(di, dj); the seven
// weights of an element add up to F.  Hence
//     contribution to a neighbour block = sum w * a_q          (only near the block's edges)
//     contribution to (I, J) itself     = F * sum a_q - (sum of the six neighbour contributions)
// and elements at least p away from every edge cost one addition.
//
// g-intervals for a local coordinate x in [0, bs): block offset -1: [x+1, p], 0: [max(x-bs+1,-p),
// min(x,p)], +1: [-p, x-bs].
//
// Fixed point in fp64: for |a| <= 1, a_q = rint((double)a * 2^40) (ties to even) is an integer of at
// most 41 bits, exact in fp64, and so are its products with the weights (< 2^7) and the sums of up
// to 64 of them that a lane forms per block (< 2^53); see the kernel.
// Build-time tunable of conv_pool_kernel: waves launched per compute unit (256 of them) at block 64; two
// per SIMD are resident.  Measured at L = 4096, block 64 (cold map, whole call): 16 (every wave one
// block) 45.0 us, 8 46.9 us, 4 49.5 us.
#ifndef SPION_CONV_WAVES_PER_CU
#define SPION_CONV_WAVES_PER_CU 16
#endif

__device__ __forceinline__ int isect(int lo_a, int hi_a, int lo_b, int hi_b) {
    const int lo = lo_a > lo_b ? lo_a : lo_b;
    const int hi = hi_a < hi_b ? hi_a : hi_b;
    const int n = hi - lo + 1;
    return n > 0 ? n : 0;
}

__device__ __forceinline__ long long shfl_xor_i64(long long v, int mask) { return __shfl_xor(v, mask); }

// Slot s of the sums of input block (I, J) belongs to pooled block (I + di(s), J + dj(s)):
// 0 (0,0)  1 (-1,0)  2 (+1,0)  3 (0,-1)  4 (0,+1)  5 (-1,-1)  6 (+1,+1)  7 unused
__device__ __forceinline__ int slot_di(int s) { return (s == 1 || s == 5) ? -1 : ((s == 2 || s == 6) ? 1 : 0); }
__device__ __forceinline__ int slot_dj(int s) { return (s == 3 || s == 5) ? -1 : ((s == 4 || s == 6) ? 1 : 0); }

// One wave per input block: the wave walks the block's 16 x 16 sub-tiles (one float4 per lane each) in
// two halves, and requests the next half (of this block or of its next block) before it works on the
// current one, so half a block's worth of loads per wave is in flight at all times.  Which neighbours
// a sub-tile can reach is known per sub-tile, so the edge work is skipped with scalar branches.  The
// wave's seven slot sums are written, without atomics, into the records of the pooled blocks they
// belong to: pooled block (ti, tj) owns the 64-byte record part[8 (ti nb + tj) .. + 7], and its slot s is
// written by exactly one input block, (ti - di(s), tj - dj(s)), if that block exists.  Nothing has to be
// zeroed beforehand.  Waves take the blocks wave_id, wave_id + n_waves, ...
template <int BS>
__global__ __launch_bounds__(256, BS == 64 ? 2 : 4) void conv_pool_kernel(const float* __restrict__ A, int L,
                                                                          int p_arg,
                                                                          long long* __restrict__ part) {
    // sub-tile of one wave instruction: SH rows x SW columns, 256 scores
    constexpr int SW = 16, SH = 256 / SW;
    constexpr int NSC = BS / SW, NSUB = (BS / SH) * NSC;
    constexpr int NH = NSUB >= 2 ? 2 : 1, HS = NSUB / NH;   // halves per block, sub-tiles per half
    const int nb = L / BS;
    const int n_blocks = nb * nb;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n_waves = gridDim.x * (blockDim.x >> 6);
    const int first = blockIdx.x * (blockDim.x >> 6) + wave;
    const int lr = lane / (SW / 4), lc = (lane % (SW / 4)) << 2;

    auto load_half = [&](int blk, int half, float4 (&dst)[HS]) {
        const float* base = A + (size_t)(blk / nb) * BS * L + (size_t)(blk % nb) * BS;
#pragma unroll
        for (int k = 0; k < HS; ++k) {
            const int st = half * HS + k;
            const int u = (st / NSC) * SH + lr, v0 = (st % NSC) * SW + lc;
            dst[k] = *reinterpret_cast<const float4*>(base + (size_t)u * L + v0);
        }
    };

    // Per lane and block the sums stay in fp64: every term is an integer (a quantised score below 2^41
    // in magnitude times a weight below 2^7), at most 64 of them go into one sum, so every partial sum
    // is an integer below 2^53 and the fp64 additions are exact.  (fp64 adds and fused multiply-adds
    // issue at the rate of fp32 ones here; the same sums in 64-bit integer arithmetic take three to
    // four instructions per term.)
    double tot[8];
    double s_all;
    // sub-tiles [half * HS, half * HS + HS) of the current block, scores in src
    auto work_half = [&](int half, const float4 (&src)[HS]) {
        // The edge weights and the coordinates they are made from depend only on the lane, the sub-tile
        // and the filter, not on the block; left to itself the compiler computes all of them once and
        // keeps several hundred values in registers (and in scratch memory) across the loop.  Hiding
        // the filter's half-width and the lane's coordinates here makes them per-sub-tile work.
#pragma unroll
        for (int k = 0; k < HS; ++k) {
            int p = p_arg, lrow = lr, lcol = lc;
            asm volatile("" : "+s"(p), "+v"(lrow), "+v"(lcol));
            __builtin_amdgcn_sched_barrier(0);   // one sub-tile at a time: their temporaries do not pile up
            const int st = half * HS + k;
            const int su = (st / NSC) * SH, sv = (st % NSC) * SW;
            const int u = su + lrow, v0 = sv + lcol;
            const bool top = su < p, bottom = su + SH - 1 > BS - 1 - p;
            const bool left = sv < p, right = sv + SW - 1 > BS - 1 - p;
            const int rm_lo = u + 1, rm_hi = p;
            const int r0_lo = (u - BS + 1) > -p ? (u - BS + 1) : -p, r0_hi = u < p ? u : p;
            const int rp_lo = -p, rp_hi = u - BS;
            const float av[4] = {src[k].x, src[k].y, src[k].z, src[k].w};
            double q[4];   // a_q = rint(a * 2^40), ties to even: an integer, exact in fp64
            int c0_lo[4], c0_hi[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int v = v0 + e;
                q[e] = __builtin_rint((double)av[e] * 1099511627776.0);
                c0_lo[e] = (v - BS + 1) > -p ? (v - BS + 1) : -p;
                c0_hi[e] = v < p ? v : p;
            }
            s_all += (q[0] + q[1]) + (q[2] + q[3]);
            auto edge = [&](int slot, auto weight) {
                double acc = tot[slot];
#pragma unroll
                for (int e = 0; e < 4; ++e) acc = __builtin_fma((double)weight(e), q[e], acc);
                tot[slot] = acc;
            };
            if (top) edge(1, [&](int e) { return isect(rm_lo, rm_hi, c0_lo[e], c0_hi[e]); });
            if (bottom) edge(2, [&](int e) { return isect(rp_lo, rp_hi, c0_lo[e], c0_hi[e]); });
            if (left) edge(3, [&](int e) { return isect(r0_lo, r0_hi, v0 + e + 1, p); });
            if (right) edge(4, [&](int e) { return isect(r0_lo, r0_hi, -p, v0 + e - BS); });
            if (top && left) edge(5, [&](int e) { return isect(rm_lo, rm_hi, v0 + e + 1, p); });
            if (bottom && right) edge(6, [&](int e) { return isect(rp_lo, rp_hi, -p, v0 + e - BS); });
        }
    };

    float4 a[HS], b[HS];
    if (first < n_blocks) load_half(first, 0, a);
    for (int blk = first; blk < n_blocks; blk += n_waves) {
        const bool more = blk + n_waves < n_blocks;
#pragma unroll
        for (int t = 0; t < 8; ++t) tot[t] = 0.0;
        s_all = 0.0;
        if constexpr (NH == 2) {
            load_half(blk, 1, b);
            work_half(0, a);
            if (more) load_half(blk + n_waves, 0, a);
            work_half(1, b);
        } else {
            if (more) load_half(blk + n_waves, 0, b);
            work_half(0, a);
#pragma unroll
            for (int k = 0; k < HS; ++k) a[k] = b[k];
        }
        // from here on in 64-bit integers: the sums over the wave's lanes can exceed 2^53
        long long ti64[8];
        long long others = 0;
#pragma unroll
        for (int t = 1; t < 7; ++t) {
            ti64[t] = (long long)tot[t];
            others += ti64[t];
        }
        ti64[0] = (long long)(2 * p_arg + 1) * (long long)s_all - others;
        ti64[7] = 0;

        // reduce-scatter butterfly over the wave: 8 slots -> 4 -> 2 -> 1, then 3 plain steps
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const bool up = lane & 32;
            const long long send = up ? ti64[k] : ti64[k + 4];
            const long long keep = up ? ti64[k + 4] : ti64[k];
            ti64[k] = keep + shfl_xor_i64(send, 32);
        }
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const bool up = lane & 16;
            const long long send = up ? ti64[k] : ti64[k + 2];
            const long long keep = up ? ti64[k + 2] : ti64[k];
            ti64[k] = keep + shfl_xor_i64(send, 16);
        }
        {
            const bool up = lane & 8;
            const long long send = up ? ti64[0] : ti64[1];
            const long long keep = up ? ti64[1] : ti64[0];
            ti64[0] = keep + shfl_xor_i64(send, 8);
        }
        long long s = ti64[0];
        s += shfl_xor_i64(s, 4);
        s += shfl_xor_i64(s, 2);
        s += shfl_xor_i64(s, 1);
        if ((lane & 7) == 0) {
            const int slot = ((lane >> 5) & 1) * 4 + ((lane >> 4) & 1) * 2 + ((lane >> 3) & 1);
            const int ti = blk / nb + slot_di(slot), tj = blk % nb + slot_dj(slot);
            if (slot < 7 && ti >= 0 && ti < nb && tj >= 0 && tj < nb) part[((size_t)ti * nb + tj) * 8 + slot] = s;
        }
    }
}

// pool_sum of cell (ti, tj): the sum of the slots of its record whose source block exists (the
// other slots were never written).
struct PoolRecord {
    uint4 q[4];
};
__device__ __forceinline__ PoolRecord load_record(const long long* __restrict__ part, size_t cell) {
    PoolRecord rec;
    const uint4* src = reinterpret_cast<const uint4*>(part + cell * 8);
#pragma unroll
    for (int h = 0; h < 4; ++h) rec.q[h] = src[h];
    return rec;
}
__device__ __forceinline__ long long sum_record(const PoolRecord& rec, int nb, int ti, int tj) {
    // slot s was written by input block (ti - di(s), tj - dj(s)): it exists iff the pooled block has a
    // neighbour on that side
    const bool up = ti >= 1, down = ti + 1 < nb, left = tj >= 1, right = tj + 1 < nb;
    const bool ok[7] = {true, down, up, right, left, down && right, up && left};
    long long acc = 0;
#pragma unroll
    for (int s = 0; s < 7; ++s) {
        const uint4 q = rec.q[s >> 1];
        const unsigned long long v = (s & 1) ? ((unsigned long long)q.w << 32 | q.z) : ((unsigned long long)q.y << 32 | q.x);
        acc += ok[s] ? (long long)v : 0ll;
    }
    return acc;
}

// pool_sum alone (the convolution + pooling stage run on its own)
__global__ __launch_bounds__(256) void pool_gather_kernel(const long long* __restrict__ part, int nb,
                                                          long long* __restrict__ pool) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < nb * nb) pool[i] = sum_record(load_record(part, (size_t)i), nb, i / nb, i % nb);
}

// ------------------------------------------------------------------------------------------------
// threshold + fill + compaction (one workgroup)
// ------------------------------------------------------------------------------------------------
constexpr int kFinishThreads = 1024;
constexpr int kFinishWaves = kFinishThreads / 64;
constexpr int SPION_MAX_NB_INTERNAL = 1024;   // same bound as SPION_MAX_NB of the public header
constexpr unsigned kDown = 1u, kRight = 2u, kDiag = 4u, kAbove = 8u;
constexpr unsigned kExpanded = 1u, kReached = 2u;

struct Thresh {
    int is_int;
    long long ti;
    double td;
};

__device__ __forceinline__ int wave_inclusive_scan(int v, int lane) {
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_up(v, off);
        if (lane >= off) v += o;
    }
    return v;
}

// The same scan with DPP moves (VALU speed, no LDS crossbar): shifts of 1, 2, 4, 8 inside each row of
// 16 lanes, then lane 15 of rows 0 and 2 added to rows 1 and 3, then lane 31 added to rows 2 and 3.
// A lane whose source is outside its row, or whose row is masked off, adds the 0 given as old value.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_fetch(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, ROW_MASK, 0xf, false);
}
__device__ __forceinline__ int wave_inclusive_scan_dpp(int v) {
    v += dpp_fetch<0x111, 0xf>(v);   // row_shr:1
    v += dpp_fetch<0x112, 0xf>(v);   // row_shr:2
    v += dpp_fetch<0x114, 0xf>(v);   // row_shr:4
    v += dpp_fetch<0x118, 0xf>(v);   // row_shr:8
    v += dpp_fetch<0x142, 0xa>(v);   // row_bcast:15 into rows 1 and 3
    v += dpp_fetch<0x143, 0xc>(v);   // row_bcast:31 into rows 2 and 3
    return v;
}

// Minimum over the wave, same data movement; the result is in lane 63.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_fetch_or_self(int v) {
    return __builtin_amdgcn_update_dpp(v, v, CTRL, ROW_MASK, 0xf, false);
}
__device__ __forceinline__ int wave_min_dpp(int v) {
    v = min(v, dpp_fetch_or_self<0x111, 0xf>(v));
    v = min(v, dpp_fetch_or_self<0x112, 0xf>(v));
    v = min(v, dpp_fetch_or_self<0x114, 0xf>(v));
    v = min(v, dpp_fetch_or_self<0x118, 0xf>(v));
    v = min(v, dpp_fetch_or_self<0x142, 0xa>(v));
    v = min(v, dpp_fetch_or_self<0x143, 0xc>(v));
    return v;
}

// Exclusive prefix sum over one value per thread.  Returns the exclusive prefix of this thread's
// value; *total gets the sum.  All threads call.  scratch: kFinishWaves + 1 ints of LDS.
__device__ int block_exclusive_scan(int v, int* total, int* scratch) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int incl = wave_inclusive_scan(v, lane);
    if (lane == 63) scratch[wave] = incl;
    __syncthreads();
    if (wave == 0) {
        const int c = lane < kFinishWaves ? scratch[lane] : 0;
        const int inc = wave_inclusive_scan(c, lane);
        if (lane < kFinishWaves) scratch[lane] = inc - c;
        if (lane == kFinishWaves - 1) scratch[kFinishWaves] = inc;
    }
    __syncthreads();
    const int res = incl - v + scratch[wave];
    *total = scratch[kFinishWaves];
    __syncthreads();
    return res;
}

// Number of kept cells in a run of nb cells starting at f with the given element stride, counted by
// one wave; with WRITE, also emits the compacted positions.
template <bool WRITE>
__device__ __forceinline__ int wave_compact(const uint8_t* f, int stride, int nb, int lane, int start,
                                            int* idx_out, int* pos_rw, long long pos_base,
                                            int pos_stride, int* bsr_pos_out) {
    int offset = start;
    for (int seg = 0; seg < nb; seg += 64) {
        const int c = seg + lane;
        const bool keep = c < nb && f[(long long)c * stride] != 0;
        const unsigned long long b = __ballot(keep);
        if (WRITE && keep) {
            const int k = offset + __popcll(b & ((1ull << lane) - 1ull));
            idx_out[k] = c;
            if (bsr_pos_out)
                bsr_pos_out[k] = pos_rw[pos_base + (long long)c * pos_stride];
            else
                pos_rw[pos_base + (long long)c * pos_stride] = k;
        }
        offset += __popcll(b);
    }
    return offset - start;
}

// Radix selection: digits of kDigitBits bits, most significant first; 64-bit keys need kSelPasses.
constexpr int kDigitBits = 11, kBins = 1 << kDigitBits, kSelPasses = 6;
static_assert(kDigitBits * (kSelPasses - 1) < 64 && kDigitBits * kSelPasses >= 64, "passes must cover 64 bits");
static_assert(kBins == 32 * 64, "one wave scans a histogram with 32 bins per lane");
// Where the counter of digit D lives in a histogram: lane D / 32 of a scanning wave owns the 32
// consecutive digits 32 (D / 32) .. + 31 as eight 16-byte groups, and group j of all lanes is
// contiguous, so that the wave reads it without bank conflicts.
__device__ __forceinline__ int bin_slot(unsigned D) { return (int)(((D >> 2) & 7u) * 256u + (D >> 5) * 4u + (D & 3u)); }

// mode: 0 = threshold given in t_abs, 1 = quantile rank k_rank, 2 = mean + kval * std.
// part: partial records of conv_pool_kernel, from which pool[] is first computed; nullptr: pool[] is given.
// mask_g / expd_g / pos: scratch arrays of nb*nb entries in global memory; when use_lds is set the
// byte arrays live in dynamic LDS instead (3 * nb * nb bytes).  mask_g holds 2 * nb * nb bytes.
__global__ __launch_bounds__(kFinishThreads) void pattern_finish_kernel(
    const long long* __restrict__ part, long long* pool, int nb, int mode, int k_rank, double kval,
    double t_abs, int no_fill, int use_lds, uint8_t* mask_g, uint8_t* expd_g, int* pos,
    uint8_t* __restrict__ fl, int* __restrict__ row_ptr, int* __restrict__ col_idx,
    int* __restrict__ col_ptr, int* __restrict__ row_idx, int* __restrict__ bsr_pos,
    int* __restrict__ nnzb_out) {
    extern __shared__ uint8_t dyn_lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = nb * nb;   // at most 2^20 cells: 32-bit index arithmetic throughout (no 64-bit divisions)
    uint8_t* mask = use_lds ? dyn_lds : mask_g;
    uint8_t* expd = use_lds ? dyn_lds + n : expd_g;
    uint8_t* mask_t = use_lds ? dyn_lds + 2 * n : mask_g + n;   // final mask, transposed (step 5)
    if (use_lds > 1) pos = reinterpret_cast<int*>(dyn_lds + 4 * n);   // 3n rounded up to a multiple of 4
    // nb <= 64: the steps after the threshold use neither expd, mask_t nor pos; pool_sum lives there
    // instead, so that the three neighbours of every cell are read from LDS
    long long* const pool_s = reinterpret_cast<long long*>(dyn_lds + ((n + 7) & ~7));
    // One block of LDS, used twice: three histograms while the quantile is selected; afterwards the
    // arrays of the fill and the compaction.
    __shared__ __attribute__((aligned(16))) unsigned char sh[3 * kBins * 4];
    unsigned* const hist = reinterpret_cast<unsigned*>(sh);
    // nb <= 64 only: successor bits of row r in anti-diagonal order, skew[r][s] = bits of cell
    // (r, s - r), zero where s - r is outside the row; the "reached" bit of every cell as one 128-bit
    // mask per row in the same order; the final mask as one 64-bit word per row and per column
    uint8_t* const skew = sh;                                                   // 64 * 128
    int* const line_start = reinterpret_cast<int*>(sh + 8192);                  // SPION_MAX_NB ints
    int* const col_start = reinterpret_cast<int*>(sh + 12288);                  // SPION_MAX_NB ints
    unsigned* const rbits = reinterpret_cast<unsigned*>(sh + 16384);            // 64 * 4
    unsigned long long* const rowmask = reinterpret_cast<unsigned long long*>(sh + 17408);   // 64
    unsigned long long* const colmask = reinterpret_cast<unsigned long long*>(sh + 17920);   // 64
    static_assert(17920 + 512 <= 3 * kBins * 4 && SPION_MAX_NB_INTERNAL * 4 == 4096, "LDS carving");
    __shared__ Thresh th;
    __shared__ int scan_scratch[kFinishWaves + 1];
    __shared__ int sel_digit, sel_below, sel_count, cand_n, common_lz;
    __shared__ unsigned long long cand[64], sel_key;
    const bool small = nb <= 64;

    // ---- 0. pool_sum from the partial records.  nb <= 64: thread (wave, lane) owns the cells
    //         (wave + 16 j, lane), j < 4, and keeps their values in registers (no division is needed to
    //         find a cell's row and column); larger grids walk the cells with a stride ------------------
    if (tid == 0) common_lz = 64;   // (read after the barrier that ends this step)
    constexpr int kCached = 4;
    static_assert(kCached * kFinishWaves == 64, "the owned cells of a thread cover 64 rows");
    auto own_cell = [&](int j, int& i) {
        const int r = wave + kFinishWaves * j;
        i = r * nb + lane;
        return r < nb && lane < nb;
    };
    long long val[kCached] = {0, 0, 0, 0};
    if (part) {
        if (small) {
            // all records are requested before the first is used
            PoolRecord rec[kCached];
#pragma unroll
            for (int j = 0; j < kCached; ++j) {
                int i;
                const bool ok = own_cell(j, i);
                rec[j] = load_record(part, (size_t)(ok ? i : 0));
            }
#pragma unroll
            for (int j = 0; j < kCached; ++j) {
                int i;
                if (own_cell(j, i)) {
                    const long long v = sum_record(rec[j], nb, wave + kFinishWaves * j, lane);
                    pool[i] = v;
                    val[j] = v;
                    pool_s[i] = v;
                }
            }
        } else {
            for (int base = 0; base < n; base += kCached * kFinishThreads) {
                PoolRecord rec[kCached];
#pragma unroll
                for (int j = 0; j < kCached; ++j) {
                    const int i = base + j * kFinishThreads + tid;
                    rec[j] = load_record(part, (size_t)(i < n ? i : n - 1));
                }
#pragma unroll
                for (int j = 0; j < kCached; ++j) {
                    const int i = base + j * kFinishThreads + tid;
                    if (i < n) pool[i] = sum_record(rec[j], nb, i / nb, i % nb);
                }
            }
        }
        __syncthreads();   // pool[] is read by other threads from here on
    } else if (small) {
#pragma unroll
        for (int j = 0; j < kCached; ++j) {
            int i;
            if (own_cell(j, i)) {
                val[j] = pool[i];
                pool_s[i] = val[j];
            }
        }
        __syncthreads();
    }

    // ---- 1. threshold ------------------------------------------------------------------------
    if (mode == 1) {
        // Exact k-th smallest (0-based) by radix selection on key = value with the sign bit flipped.
        // A pass: every wave counts its keys' digits into a histogram; one wave scans it (32 bins per
        // lane, a DPP prefix sum) and publishes the digit that holds rank k; three histograms rotate,
        // the other waves clear the one of the pass before meanwhile.
        for (int i = tid; i < 3 * kBins; i += kFinishThreads) hist[i] = 0u;
        if (tid == 0) cand_n = 0;
        unsigned long long key[kCached];
        bool alive[kCached];   // still equal to the selected prefix
        // The leading bits that all keys share need no pass: pooled sums of scores in [0, 1] share their
        // first 14 bits or more.  Every key is compared with the key of cell (0, 0); the smallest number
        // of leading bits any key shares with it is what all keys share.  (nb <= 64 only.)
        const unsigned long long ref = small ? ((unsigned long long)pool_s[0] ^ 0x8000000000000000ull) : 0ull;
        unsigned long long differ = 0ull;
#pragma unroll
        for (int j = 0; j < kCached; ++j) {
            key[j] = (unsigned long long)val[j] ^ 0x8000000000000000ull;
            int i;
            alive[j] = small && own_cell(j, i);
            if (alive[j]) differ |= key[j] ^ ref;
        }
        if (small) {
            const int lz = wave_min_dpp(differ ? __clzll((long long)differ) : 64);
            if (lane == 63) atomicMin(&common_lz, lz);
        }
        __syncthreads();
        const int shared_bits = small ? common_lz : 0;
        const int n_passes = (64 - shared_bits + kDigitBits - 1) / kDigitBits;   // 0: all keys are equal
        unsigned long long prefix = 0ull;
        if (small && kDigitBits * n_passes < 64) prefix = ref & ~((1ull << (kDigitBits * n_passes)) - 1ull);
        int k = k_rank;
#pragma unroll 1
        for (int pass = 0; pass < n_passes; ++pass) {
            const int shift = kDigitBits * (n_passes - 1 - pass);   // without shared bits: 55, 44, ..., 0
            const int top = shift + kDigitBits;                     // bits >= top are already decided
            unsigned* const h = hist + (pass % 3) * kBins;
            auto count = [&](unsigned long long u, bool match) {
                const unsigned digit = (unsigned)(u >> shift) & (unsigned)(kBins - 1);
                // the leading digits are usually equal for the whole wave: one atomic instead of 64
                const unsigned long long m = __ballot(match);
                if (m == 0ull) return;
                const unsigned first = (unsigned)__builtin_amdgcn_readlane((int)digit, __ffsll((long long)m) - 1);
                if (__ballot(match && digit == first) == m) {
                    if (lane == 0) atomicAdd(&h[bin_slot(first)], (unsigned)__popcll(m));
                } else if (match) {
                    atomicAdd(&h[bin_slot(digit)], 1u);
                }
            };
            if (small) {
#pragma unroll
                for (int j = 0; j < kCached; ++j) count(key[j], alive[j]);
            } else {
                for (int base = 0; base < n; base += kFinishThreads) {
                    const int i = base + tid;
                    const unsigned long long u =
                        i < n ? ((unsigned long long)pool[i] ^ 0x8000000000000000ull) : 0ull;
                    count(u, i < n && (top >= 64 || (u >> top) == (prefix >> top)));
                }
            }
            __syncthreads();
            if (wave != 0) {
                // the histogram of the pass before (last read before the barrier above) is cleared for the
                // pass after the next, off the path of the wave that scans
                unsigned* const hz = hist + ((pass + 2) % 3) * kBins;
                for (int i = tid - 64; i < kBins; i += kFinishThreads - 64) hz[i] = 0u;
            } else {
                // the digit whose bin holds rank k: lane owns digits 32 lane .. 32 lane + 31 as 8 groups of 4
                const uint4* const h4 = reinterpret_cast<const uint4*>(h);
                int s4[8], s32 = 0;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const uint4 v = h4[j * 64 + lane];
                    s4[j] = (int)(v.x + v.y + v.z + v.w);
                    s32 += s4[j];
                }
                const int incl = wave_inclusive_scan_dpp(s32);
                int e = incl - s32, qj = 0;
                const bool hit = k >= e && k < incl;   // exactly one lane: the matching keys number more than k
#pragma unroll
                for (int j = 0; j < 7; ++j) {
                    const bool adv = qj == j && k >= e + s4[j];
                    e = adv ? e + s4[j] : e;
                    qj = adv ? j + 1 : qj;
                }
                const uint4 v = h4[qj * 64 + lane];
                const int c3[3] = {(int)v.x, (int)v.y, (int)v.z};
                int qt = 0;
#pragma unroll
                for (int j = 0; j < 3; ++j) {
                    const bool adv = qt == j && k >= e + c3[j];
                    e = adv ? e + c3[j] : e;
                    qt = adv ? j + 1 : qt;
                }
                if (hit) {
                    sel_digit = 32 * lane + 4 * qj + qt;
                    sel_below = e;   // matching keys below that digit
                    sel_count = (int)(qt == 0 ? v.x : (qt == 1 ? v.y : (qt == 2 ? v.z : v.w)));   // matching keys with that digit
                }
            }
            __syncthreads();
            const unsigned digit = (unsigned)sel_digit;
            k -= sel_below;
            prefix |= (unsigned long long)digit << shift;
#pragma unroll
            for (int j = 0; j < kCached; ++j)
                alive[j] = alive[j] && ((unsigned)(key[j] >> shift) & (unsigned)(kBins - 1)) == digit;
            if (pass + 1 < n_passes && sel_count <= 64) {
                // Few keys are left (typically after the third pass): instead of the remaining passes they
                // are collected and one wave ranks them against each other.  k is the rank among them.
                if (small) {
#pragma unroll
                    for (int j = 0; j < kCached; ++j)
                        if (alive[j]) cand[atomicAdd(&cand_n, 1)] = key[j];
                } else {
                    for (int base = 0; base < n; base += kFinishThreads) {
                        const int i = base + tid;
                        if (i < n) {
                            const unsigned long long u = (unsigned long long)pool[i] ^ 0x8000000000000000ull;
                            if ((u >> shift) == (prefix >> shift)) cand[atomicAdd(&cand_n, 1)] = u;
                        }
                    }
                }
                __syncthreads();
                if (wave == 0) {
                    const int cn = cand_n;   // == sel_count
                    const unsigned long long mine = lane < cn ? cand[lane] : ~0ull;
                    int less = 0, same = 0;
                    for (int t = 0; t < cn; ++t) {
                        const unsigned long long other = cand[t];
                        less += other < mine ? 1 : 0;
                        same += other == mine ? 1 : 0;
                    }
                    if (lane < cn && k >= less && k < less + same) sel_key = mine;   // equal keys write the same value
                }
                __syncthreads();
                prefix = sel_key;
                break;
            }
        }
        if (tid == 0) {
            th.is_int = 1;
            th.ti = (long long)(prefix ^ 0x8000000000000000ull);
            th.td = (double)th.ti;
        }
    } else if (mode == 2) {
        // sequential fp64 sums in row-major order: this is the definition, not an optimisation target
        if (tid == 0) {
            double sum = 0.0;
            for (int i = 0; i < n; ++i) sum = sum + (double)pool[i];
            const double mean = sum / (double)n;
            double ss = 0.0;
            for (int i = 0; i < n; ++i) {
                const double dlt = (double)pool[i] - mean;
                const double sq = dlt * dlt;
                ss = ss + sq;
            }
            const double var = ss / (double)n;
            const double sd = sqrt(var);
            const double ks = kval * sd;
            th.is_int = 0;
            th.ti = 0;
            th.td = mean + ks;
        }
    } else {
        if (tid == 0) {
            th.is_int = 0;
            th.ti = 0;
            th.td = t_abs;
        }
    }
    __syncthreads();
    const Thresh t = th;
    if (small) {
        // the histograms are done with: their LDS now holds the arrays of the steps below
        for (int i = tid; i < 64 * 128 / 4; i += kFinishThreads) reinterpret_cast<unsigned*>(skew)[i] = 0u;
        __syncthreads();
    }

    // ---- 2. per cell: successor bits (which of down / right / diag equal their maximum), the
    //         "above threshold" bit, and the seed flag (first row and first column) ------------------
    auto cell_bits = [&](long long x, long long dn, long long rt, long long dg, bool inner) {
        bool ab;
        if (t.is_int) ab = x > t.ti;
        else ab = (double)x > t.td;
        unsigned m = ab ? kAbove : 0u;
        if (inner) {
            long long mx = dn > rt ? dn : rt;
            mx = mx > dg ? mx : dg;
            m |= (dn == mx ? kDown : 0u) | (rt == mx ? kRight : 0u) | (dg == mx ? kDiag : 0u);
        }
        return m;
    };
    if (small) {
#pragma unroll
        for (int j = 0; j < kCached; ++j) {
            int i;
            if (!own_cell(j, i)) continue;
            const int r = wave + kFinishWaves * j, c = lane;
            const bool inner = r + 1 < nb && c + 1 < nb;
            long long dn = 0, rt = 0, dg = 0;
            if (inner) {
                dn = pool_s[i + nb];
                rt = pool_s[i + 1];
                dg = pool_s[i + nb + 1];
            }
            const unsigned m = cell_bits(val[j], dn, rt, dg, inner);
            mask[i] = (uint8_t)m;
            skew[r * 128 + r + c] = (uint8_t)(m & 7u);
        }
    } else {
        for (int i = tid; i < n; i += kFinishThreads) {
            const int r = i / nb, c = i % nb;
            const bool inner = r + 1 < nb && c + 1 < nb;
            long long dn = 0, rt = 0, dg = 0;
            if (inner) {
                dn = pool[i + nb];
                rt = pool[i + 1];
                dg = pool[i + nb + 1];
            }
            mask[i] = (uint8_t)cell_bits(pool[i], dn, rt, dg, inner);
            expd[i] = no_fill ? (uint8_t)kReached : ((r == 0 || c == 0) ? (uint8_t)kExpanded : (uint8_t)0);
        }
    }
    __syncthreads();

    // ---- 3. fill: every move raises r + c, so anti-diagonal s depends only on s-1 and s-2.  A cell is
    //         reached iff an expanded predecessor lists it as a successor; reached cells are expanded
    //         in turn whether or not they exceed the threshold. -------------------------------------
    if (!no_fill) {
        if (small) {
            // One wave, lane = row r.  The row's successor bits sit in 32 registers in anti-diagonal
            // order, so level s reads a compile-time register; the outgoing bits of the previous
            // two levels travel in registers and the neighbour row's bits arrive by a one-lane
            // shift.  Cells outside the matrix have no bits and can neither be reached nor expand.
            if (wave == 0) {
                const int r = lane;
                unsigned sk[32];
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const uint4 v = reinterpret_cast<const uint4*>(skew + r * 128)[q];
                    sk[4 * q] = v.x;
                    sk[4 * q + 1] = v.y;
                    sk[4 * q + 2] = v.z;
                    sk[4 * q + 3] = v.w;
                }
                unsigned out1 = 0u, out2 = 0u;
                unsigned rb[4] = {0u, 0u, 0u, 0u};
#pragma unroll
                for (int s = 0; s < 127; ++s) {
                    const unsigned m = (sk[s >> 2] >> (8 * (s & 3))) & 7u;
                    const unsigned both = out1 | (out2 << 8);
                    const unsigned up = __builtin_amdgcn_update_dpp(0u, both, 0x138 /* wave_shr:1 */,
                                                                    0xf, 0xf, false);
                    const unsigned hit = (out1 & kRight) | (up & kDown) | ((up >> 8) & kDiag);
                    const bool reached = hit != 0u;
                    const bool expanded = reached || r == 0 || s == r;   // seeds: row 0, column 0
                    rb[s >> 5] |= (reached ? 1u : 0u) << (s & 31);
                    out2 = out1;
                    out1 = expanded ? m : 0u;
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) rbits[r * 4 + q] = rb[q];
            }
        } else {
            for (int s = 1; s <= 2 * nb - 2; ++s) {
                const int r = tid, c = s - tid;
                if (r < nb && c >= 0 && c < nb) {
                    const int i = r * nb + c;
                    bool reached = false;
                    if (r >= 1) reached |= (expd[i - nb] & kExpanded) && (mask[i - nb] & kDown);
                    if (c >= 1) reached |= (expd[i - 1] & kExpanded) && (mask[i - 1] & kRight);
                    if (r >= 1 && c >= 1)
                        reached |= (expd[i - nb - 1] & kExpanded) && (mask[i - nb - 1] & kDiag);
                    if (reached) expd[i] = (uint8_t)(kExpanded | kReached);
                }
                __syncthreads();
            }
        }
    }
    __syncthreads();
    const bool want_bsc = col_ptr != nullptr;

    if (small) {
        // ---- 4 + 5, nb <= 64: the final mask as one 64-bit word per row (a wave's ballot over the
        //      row's cells) and per column; every kept cell then finds its place in BSR and BSC from
        //      population counts of those words, with no pass over the matrix in between -------------
        auto kept = [&](int r, int c) {
            if (c >= nb) return false;
            const bool reached = no_fill || ((rbits[r * 4 + ((r + c) >> 5)] >> ((r + c) & 31)) & 1u) != 0u;
            return (reached && (mask[r * nb + c] & kAbove)) || r == c;
        };
        for (int r = wave; r < nb; r += kFinishWaves) {
            const bool f = kept(r, lane);
            if (lane < nb) fl[r * nb + lane] = f ? 1 : 0;
            const unsigned long long m = __ballot(f);
            if (lane == 0) rowmask[r] = m;
        }
        __syncthreads();
        {
            // the column words: lane r holds row r's word, a ballot over bit c is column c; wave w makes the
            // columns w, w + 16, ...
            const unsigned long long rm = lane < nb ? rowmask[lane] : 0ull;
            for (int c = wave; c < nb; c += kFinishWaves) {
                const unsigned long long cm = __ballot(((rm >> c) & 1ull) != 0ull);
                if (lane == 0) colmask[c] = cm;
            }
        }
        __syncthreads();
        if (wave == 0) {
            const int v = lane < nb ? __popcll(rowmask[lane]) : 0;
            const int incl = wave_inclusive_scan_dpp(v);
            if (lane < nb) {
                line_start[lane] = incl - v;
                row_ptr[lane] = incl - v;
            }
            if (lane == 63) {
                row_ptr[nb] = incl;
                *nnzb_out = incl;
            }
        } else if (wave == 1 && want_bsc) {
            const int v = lane < nb ? __popcll(colmask[lane]) : 0;
            const int incl = wave_inclusive_scan_dpp(v);
            if (lane < nb) {
                col_start[lane] = incl - v;
                col_ptr[lane] = incl - v;
            }
            if (lane == 63) col_ptr[nb] = incl;
        }
        __syncthreads();
        for (int r = wave; r < nb; r += kFinishWaves) {
            const int c = lane;
            const unsigned long long rm = rowmask[r];
            if (c < nb && ((rm >> c) & 1ull)) {
                const int k = line_start[r] + __popcll(rm & ((1ull << c) - 1ull));
                col_idx[k] = c;
                if (want_bsc) {
                    const int k2 = col_start[c] + __popcll(colmask[c] & ((1ull << r) - 1ull));
                    row_idx[k2] = r;
                    bsr_pos[k2] = k;
                }
            }
        }
        return;
    }

    // ---- 4. fl_out = reached and above the threshold, or on the diagonal; kept in expd for step 5 ---
    for (int i = tid; i < n; i += kFinishThreads) {
        const int r = i / nb, c = i % nb;
        const bool reached = (expd[i] & kReached) != 0;
        const uint8_t f = ((reached && (mask[i] & kAbove)) || r == c) ? 1 : 0;
        fl[i] = f;
        mask[i] = f;
        mask_t[(long long)c * nb + r] = f;
    }
    __syncthreads();

    // ---- 5. compaction: BSR (rows) and BSC (columns); one wave per row / column -------------------
    for (int r = wave; r < nb; r += kFinishWaves) {
        const int k = wave_compact<false>(mask + (long long)r * nb, 1, nb, lane, 0, nullptr, nullptr, 0, 0,
                                          nullptr);
        if (lane == 0) line_start[r] = k;
        if (want_bsc) {
            const int kc = wave_compact<false>(mask_t + (long long)r * nb, 1, nb, lane, 0, nullptr, nullptr,
                                               0, 0, nullptr);
            if (lane == 0) col_start[r] = kc;
        }
    }
    __syncthreads();
    {
        int total = 0;
        int cnt = tid < nb ? line_start[tid] : 0;   // nb <= 1024 == kFinishThreads
        int start = block_exclusive_scan(cnt, &total, scan_scratch);
        if (tid < nb) {
            line_start[tid] = start;
            row_ptr[tid] = start;
        }
        if (tid == 0) {
            row_ptr[nb] = total;
            *nnzb_out = total;
        }
        if (want_bsc) {
            cnt = tid < nb ? col_start[tid] : 0;
            start = block_exclusive_scan(cnt, &total, scan_scratch);
            if (tid < nb) {
                col_start[tid] = start;
                col_ptr[tid] = start;
            }
            if (tid == 0) col_ptr[nb] = total;
        }
        __syncthreads();
    }
    for (int r = wave; r < nb; r += kFinishWaves)
        wave_compact<true>(mask + (long long)r * nb, 1, nb, lane, line_start[r], col_idx, pos,
                           (long long)r * nb, 1, nullptr);
    if (want_bsc) {
        __syncthreads();   // pos[] of every kept cell is written
        for (int c = wave; c < nb; c += kFinishWaves)
            wave_compact<true>(mask_t + (long long)c * nb, 1, nb, lane, col_start[c], row_idx, pos,
                               (long long)c, nb, bsr_pos);
    }
}

// ------------------------------------------------------------------------------------------------
// index check (one workgroup)
// ------------------------------------------------------------------------------------------------
// The attention kernels trust their index: an entry out of range there is an access out of bounds.
// An index that did not come from pattern_finish_kernel can be checked here first.  Three stages,
// each reading only what the stage before has shown to be in range: (1) the pointer arrays run
// from 0 to nnzb without decreasing; (2) the entries of every row (column) lie in [0, nb) and
// ascend strictly; (3) every entry of the transposed index names a position of the row-wise index
// that lies in the row it claims and holds the column it claims (with equal counts and distinct
// (row, column) pairs, that makes the transposed index the exact transpose).
__global__ __launch_bounds__(1024) void index_check_kernel(
    const int* __restrict__ row_ptr, const int* __restrict__ col_idx, const int* __restrict__ col_ptr,
    const int* __restrict__ row_idx, const int* __restrict__ bsr_pos, int nb, int nnzb, int err_code,
    int* __restrict__ status) {
    __shared__ int bad;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n_waves = blockDim.x >> 6;
    if (tid == 0) bad = 0;
    __syncthreads();
    auto pointers_ok = [&](const int* ptr) {
        bool ok = true;
        for (int i = tid; i < nb; i += blockDim.x) {
            const int a = ptr[i], b = ptr[i + 1];
            ok = ok && a >= 0 && b >= a && b <= nnzb;
        }
        if (tid == 0) ok = ok && ptr[0] == 0 && ptr[nb] == nnzb;
        return ok;
    };
    if (!pointers_ok(row_ptr)) bad = 1;
    if (col_ptr && !pointers_ok(col_ptr)) bad = 1;
    __syncthreads();
    if (bad) {
        if (tid == 0) *status = err_code;
        return;
    }
    auto entries_ok = [&](const int* ptr, const int* idx) {
        bool ok = true;
        for (int i = wave; i < nb; i += n_waves) {
            const int a = ptr[i], b = ptr[i + 1];
            for (int k = a + lane; k < b; k += 64) {
                const int c = idx[k];
                ok = ok && c >= 0 && c < nb && (k == a || idx[k - 1] < c);
            }
        }
        return ok;
    };
    if (!entries_ok(row_ptr, col_idx)) bad = 1;
    if (col_ptr && !entries_ok(col_ptr, row_idx)) bad = 1;
    __syncthreads();
    if (bad) {
        if (tid == 0) *status = err_code;
        return;
    }
    if (col_ptr) {
        bool ok = true;
        for (int j = wave; j < nb; j += n_waves) {
            const int a = col_ptr[j], b = col_ptr[j + 1];
            for (int k = a + lane; k < b; k += 64) {
                const int i = row_idx[k], pos = bsr_pos[k];
                ok = ok && pos >= row_ptr[i] && pos < row_ptr[i + 1] && col_idx[pos] == j;
            }
        }
        if (!ok) bad = 1;
    }
    __syncthreads();
    if (tid == 0) *status = bad ? err_code : 0;
}

// ------------------------------------------------------------------------------------------------
// host launchers
// ------------------------------------------------------------------------------------------------
hipError_t launch_conv_pool(const float* A, int L, int bs, int p, long long* part, hipStream_t st) {
    const int nb = L / bs;
    const unsigned blocks = (unsigned)nb * (unsigned)nb;
    // SPION_CONV_WAVES_PER_CU waves per compute unit (256 of them) at block 64, each walking several
    // input blocks; smaller blocks are fewer bytes per wave, so proportionally more waves
    auto grid = [&](unsigned waves_per_cu) {
        const unsigned wgs = (blocks + 3) / 4, cap = 256u * waves_per_cu / 4;
        return dim3(wgs < cap ? wgs : cap);
    };
    if (bs == 16)
        conv_pool_kernel<16><<<grid(4 * SPION_CONV_WAVES_PER_CU), dim3(256), 0, st>>>(A, L, p, part);
    else if (bs == 32)
        conv_pool_kernel<32><<<grid(2 * SPION_CONV_WAVES_PER_CU), dim3(256), 0, st>>>(A, L, p, part);
    else
        conv_pool_kernel<64><<<grid(SPION_CONV_WAVES_PER_CU), dim3(256), 0, st>>>(A, L, p, part);
    return hipGetLastError();
}

hipError_t launch_pool_gather(const long long* part, int nb, long long* pool, hipStream_t st) {
    pool_gather_kernel<<<dim3((unsigned)((nb * nb + 255) / 256)), dim3(256), 0, st>>>(part, nb, pool);
    return hipGetLastError();
}

hipError_t launch_pattern_finish(const long long* part, long long* pool, int nb, int mode, long long k_rank,
                                 double kval, double t_abs, int no_fill, uint8_t* mask, uint8_t* expd, int* pos,
                                 uint8_t* fl, int* row_ptr, int* col_idx, int* col_ptr, int* row_idx,
                                 int* bsr_pos, int* nnzb, hipStream_t st) {
    const size_t n = (size_t)nb * nb;
    // keep static (~25 KB) + dynamic LDS under 64 KB: the three byte arrays if 3n fits, and the
    // position array (4n more, placed at offset 4n) if 8n fits as well
    const int use_lds = 8 * n <= 36 * 1024 ? 2 : (3 * n <= 36 * 1024 ? 1 : 0);
    // nb <= 64: the byte map and, 8-byte aligned behind it, pool_sum itself (36 KB at nb = 64)
    const size_t dyn = nb <= 64 ? ((n + 7) & ~(size_t)7) + 8 * n : (use_lds == 2 ? 8 * n : (use_lds == 1 ? 3 * n : 0));
    pattern_finish_kernel<<<dim3(1), dim3(kFinishThreads), dyn, st>>>(
        part, pool, nb, mode, (int)k_rank, kval, t_abs, no_fill, use_lds, mask, expd, pos, fl, row_ptr, col_idx,
        col_ptr, row_idx, bsr_pos, nnzb);
    return hipGetLastError();
}

hipError_t launch_index_check(const int* row_ptr, const int* col_idx, const int* col_ptr, const int* row_idx,
                              const int* bsr_pos, int nb, int nnzb, int err_code, int* status, hipStream_t st) {
    index_check_kernel<<<dim3(1), dim3(1024), 0, st>>>(row_ptr, col_idx, col_ptr, row_idx, bsr_pos, nb, nnzb,
                                                       err_code, status);
    return hipGetLastError();
}

}  // namespace spion
