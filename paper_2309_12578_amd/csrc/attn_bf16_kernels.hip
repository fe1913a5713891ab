// bf16 block-sparse attention kernels tuned for gfx950, block size 32 or 64.
//
// Same mathematics and wave tiling as the generic kernels (16 owned rows per wave on the N index of
// every MFMA tile), plus:
//   - tiles travel HBM -> LDS through the memory pipeline (global_load_lds), one to two blocks
//     ahead of the block being multiplied: no staging registers, no LDS stores, one barrier per
//     kept block;
//   - tiles stay row-major in LDS, 16-byte slots permuted per row so that no read conflicts;
//     operands that must be read along the row index (V for O = P V, K for dQ, Q and dO for
//     dK / dV) come out of the same tile through the LDS transpose read (ds_read_b64_tr_b16:
//     16 lanes fetch a 4 x 16 patch and each receives one column of it);
//   - the row-walking kernels start loading the diagonal block before they have read the index;
//   - workgroup ids are remapped so that each of the 8 XCDs (one L2 each) works on whole heads.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "attn_common.h"
#include "spion_internal.h"

namespace spion {

// Developer build only (-DSPION_KERNEL_TRACE): workgroup timestamps of pipeline stages, 16 slots per
// workgroup, written to a buffer the test harness installs with hipMemcpyToSymbol.
#ifdef SPION_KERNEL_TRACE
__device__ long long* spion_trace_buf = nullptr;
void set_trace_buf(long long* p) { (void)hipMemcpyToSymbol(HIP_SYMBOL(spion_trace_buf), &p, sizeof(p)); }
#define SPION_TP(slot)                                                                          \
    do {                                                                                        \
        if (threadIdx.x == 0 && spion_trace_buf) spion_trace_buf[(size_t)blockIdx.x * 16 + (slot)] = wall_clock64(); \
    } while (0)
#else
#define SPION_TP(slot) do { } while (0)
#endif

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

// ------------------------------------------------------------------------------------------------
// forward and backward query side: K / V tiles in two LDS stages, the next block loading while the
// current one is multiplied.  Two stages of {K, V} are 32 KB at block 64; four workgroups share a CU
// with up to 40 KB each.  (A third stage is 48 KB, i.e. three workgroups per CU, and measured 5-10 %
// slower; three K stages + two V stages with a second barrier per block measured 4 % slower.)
// ------------------------------------------------------------------------------------------------
template <int BS>
struct KvSmem {
    bf16_t k[BS * kD];
    bf16_t v[BS * kD];
};

// Wait until this wave's loads of the current block have landed, then meet the other waves: their
// parts have landed too and nobody reads the other stage any more.  younger_in_flight: the block
// after this one was already requested (only at step 0, from the prologue) and may stay in flight.
// A bare barrier: __syncthreads adds fences the kernel has no use for.
__device__ __forceinline__ void stage_ready(bool younger_in_flight) {
    if (younger_in_flight) __builtin_amdgcn_s_waitcnt(kWaitVm4);
    else __builtin_amdgcn_s_waitcnt(kWaitVm0);
    __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
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

template <int BS>
__global__ __launch_bounds__(BS * 4) void attn_fwd_bf16_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    bf16_t* __restrict__ O, float* __restrict__ LSE, const int* __restrict__ row_ptr,
    const int* __restrict__ col_idx, int L, int nb, int total, float scale_log2, int paper_denom) {
    constexpr int NKT = BS / 16;
    __shared__ __attribute__((aligned(16))) KvSmem<BS> sm0, sm1;
    SPION_TP(0);

    const int vid = xcd_remap(blockIdx.x, total);
    const int I = vid % nb, bh = vid / nb;
    const int tid = threadIdx.x, lane = tid & 63, r = lane & 15, g = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const size_t head = (size_t)bh * L * kD;
    const int qrow = I * BS + wave * 16 + r;
    const SwzLane sl(r, g);
    const TileLoadLane tl(wave, lane);

    auto issue = [&](KvSmem<BS>& st, int J) {
        tile_load_async(K + head + (size_t)J * BS * kD, st.k, wave, tl);
        tile_load_async(V + head + (size_t)J * BS * kD, st.v, wave, tl);
    };
    issue(sm0, I);   // the diagonal block, before any index is known
    bf16x8 qf[2];
#pragma unroll
    for (int c = 0; c < 2; ++c)
        qf[c] = *reinterpret_cast<const bf16x8*>(Q + head + (size_t)qrow * kD + c * 32 + g * 8);
    const int jb = row_ptr[I], n = row_ptr[I + 1] - jb;
    const int last = n > 0 ? n - 1 : 0;
    const int* cols = col_idx + jb;
    int first[8];
    const int pd = n > 0 ? find_in_row(cols, n, I, first) : -1;
    // block visited at step t (clamped reads stay inside this row's entries; an empty row reads nothing)
    auto col_at = [&](int t) {
        const int j = walk_index(t < last ? t : last, pd);
        return j < 8 ? pick8(first, j) : cols[j];
    };
    if (pd < 0 && n > 0) {
        // no diagonal block in this row: once everyone's early load has landed, load block 0 over it
        __builtin_amdgcn_s_waitcnt(kWaitVm0);
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        issue(sm0, first[0]);
    }
    // the second block goes out as soon as its index is known; it is the youngest load from here on
    if (n > 0) issue(sm1, col_at(1));   // (a one-block row loads its block twice: keeps the wait below uniform)
    int Jnext = n > 0 ? col_at(2) : 0;   // block of step it + 1, for it >= 1

    float m = -INFINITY;   // running row maximum in log2 units (score * scale * log2 e)
    f32x4 lacc = f32x4{0.f, 0.f, 0.f, 0.f};   // running row sum, replicated in its 4 elements
    f32x4 oacc[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) oacc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    bf16x8 ones;
#pragma unroll
    for (int e = 0; e < 8; ++e) ones[e] = (bf16_t)1.0f;

    auto step = [&](const KvSmem<BS>& cur, KvSmem<BS>& tgt, int it) {
        if (it < 6) SPION_TP(2 + 2 * it);
        // loads in flight here: block `it`, and at step 0 also block 1, requested by the prologue (the
        // four youngest loads: whatever else the prologue stored or loaded after them only adds waiting)
        stage_ready(it == 0);
        if (it < 6) SPION_TP(3 + 2 * it);
        if (it > 0) {
            if (it + 1 < n) issue(tgt, Jnext);
            Jnext = col_at(it + 2);
        }
        // S^T tile kt: [key 16 kt + 4 g + i][query r]
        f32x4 s[NKT];
        float mx = -INFINITY;
#pragma unroll
        for (int kt = 0; kt < NKT; ++kt) {
            s[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int c = 0; c < 2; ++c)
                s[kt] = mma_d(s[kt], *reinterpret_cast<const bf16x8*>(cur.k + kt * 16 * kD + sl.frag[c]), qf[c]);
#pragma unroll
            for (int i = 0; i < 4; ++i) mx = fmaxf(mx, s[kt][i]);
        }
        mx = group_max(mx);
        const float m_new = fmaxf(m, mx * scale_log2);
        if (__any(m_new > m)) {   // some row's running maximum moved: rescale what is accumulated
            const float alpha = fast_exp2(m - m_new);
            lacc *= alpha;
#pragma unroll
            for (int dt = 0; dt < 4; ++dt) oacc[dt] *= alpha;
        }
        bf16x4 pq[NKT];
#pragma unroll
        for (int kt = 0; kt < NKT; ++kt) {
#pragma unroll
            for (int i = 0; i < 4; ++i) s[kt][i] = fast_exp2(fmaf(s[kt][i], scale_log2, -m_new));
            pq[kt] = to_quad<bf16_t>(s[kt]);
        }
        // row sums on the MFMA pipe: a tile of ones times P^T adds up each owned row's probabilities
        // (the bf16 values that also enter P V), every accumulator element holding the same sum
#pragma unroll
        for (int pc = 0; pc < BS / 32; ++pc) lacc = mma_d(lacc, ones, join(pq[2 * pc], pq[2 * pc + 1]));
        m = m_new;
        mma_over_rows_swz<BS>(oacc, cur.v, pq, sl);   // O^T[d][query] += V^T P^T
    };

    for (int it = 0; it < n; it += 2) {
        step(sm0, sm1, it);
        if (it + 1 < n) step(sm1, sm0, it + 1);
    }

    // an empty row never waited for its early load: it must land before this workgroup's LDS is freed
    __builtin_amdgcn_s_waitcnt(kWaitVm0);

    float lsum = lacc[0];
    if (paper_denom && n > 0) {
        // Algorithm 6: every masked entry of the row counts as a score of 0 (a row that keeps nothing
        // has no entry to normalise and stays at O = 0, LSE = -inf)
        const float masked = (float)(L - n * BS);
        const float mp = fmaxf(m, 0.f);
        const float a = exp2f(m - mp);
        lsum = lsum * a + masked * exp2f(-mp);
        m = mp;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) oacc[dt] *= a;
    }
    const float inv = lsum > 0.f ? 1.f / lsum : 0.f;
    SPION_TP(14);
    // the stage that the last block did not use is free: every wave is past the barrier that followed
    // its last reader, and the only load that ever targets this wave's 2 KB of it was the wave's own
    bf16_t* patch = ((n & 1) ? sm1.k : sm0.k) + wave * (16 * kD);
    store_rows_coalesced(patch, O + head + (size_t)(I * BS + wave * 16) * kD, oacc, inv, lane);
    if (g == 0) LSE[(size_t)bh * L + qrow] = lsum > 0.f ? (m + log2f(lsum)) * kLn2 : -INFINITY;
    SPION_TP(15);
}

template <int BS>
__global__ __launch_bounds__(BS * 4) void attn_bwd_dq_bf16_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const bf16_t* __restrict__ O, const bf16_t* __restrict__ dO, const float* __restrict__ LSE,
    bf16_t* __restrict__ dQ, float* __restrict__ delta_out, float* __restrict__ lse2_out,
    const int* __restrict__ row_ptr,
    const int* __restrict__ col_idx, const int* __restrict__ col_ptr, const int* __restrict__ row_idx,
    int w_max, int split_max, int4* __restrict__ sched, int4* __restrict__ split, int L, int nb, int total,
    float scale, float scale_log2) {
    constexpr int NKT = BS / 16;
    __shared__ __attribute__((aligned(16))) KvSmem<BS> sm0, sm1;

    const int vid = xcd_remap(blockIdx.x, total);
    const int I = vid % nb, bh = vid / nb;
    const int tid = threadIdx.x, lane = tid & 63, r = lane & 15, g = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const size_t head = (size_t)bh * L * kD;
    const int qrow = I * BS + wave * 16 + r;
    const SwzLane sl(r, g);
    const TileLoadLane tl(wave, lane);

    auto issue = [&](KvSmem<BS>& st, int J) {
        tile_load_async(K + head + (size_t)J * BS * kD, st.k, wave, tl);
        tile_load_async(V + head + (size_t)J * BS * kD, st.v, wave, tl);
    };
    issue(sm0, I);   // the diagonal block, before any index is known
    bf16x8 qf[2], dof[2], of[2];
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const size_t off = head + (size_t)qrow * kD + c * 32 + g * 8;
        qf[c] = *reinterpret_cast<const bf16x8*>(Q + off);
        dof[c] = *reinterpret_cast<const bf16x8*>(dO + off);
        of[c] = *reinterpret_cast<const bf16x8*>(O + off);
    }
    const float lse2 = LSE[(size_t)bh * L + qrow] * kLog2e;
    const int jb = row_ptr[I], n = row_ptr[I + 1] - jb;
    const int last = n > 0 ? n - 1 : 0;
    const int* cols = col_idx + jb;
    int first[8];
    const int pd = n > 0 ? find_in_row(cols, n, I, first) : -1;
    // block visited at step t (clamped reads stay inside this row's entries; an empty row reads nothing)
    auto col_at = [&](int t) {
        const int j = walk_index(t < last ? t : last, pd);
        return j < 8 ? pick8(first, j) : cols[j];
    };
    if (pd < 0 && n > 0) {
        // no diagonal block in this row: once everyone's early load has landed, load block 0 over it
        __builtin_amdgcn_s_waitcnt(kWaitVm0);
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        issue(sm0, first[0]);
    }
    // the second block goes out as soon as its index is known
    if (n > 0) issue(sm1, col_at(1));   // (a one-block row loads its block twice: keeps the wait below uniform)
    int Jnext = n > 0 ? col_at(2) : 0;   // block of step it + 1, for it >= 1

    if (vid == 0 && tid < 64) build_key_schedule(col_ptr, row_idx, nb, w_max, split_max, sched, split, tid);

    float delta = 0.f;
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int e = 0; e < 8; ++e) delta = fmaf((float)dof[c][e], (float)of[c][e], delta);
    delta = group_sum(delta);
    if (g == 0) {
        delta_out[(size_t)bh * L + qrow] = -delta;   // stored negated: it seeds the dP accumulators
        lse2_out[(size_t)bh * L + qrow] = lse2;   // LSE in log2 units: the key side needs no multiply
    }

    f32x4 dq[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) dq[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto step = [&](const KvSmem<BS>& cur, KvSmem<BS>& tgt, int it) {
        stage_ready(it == 0);   // see the forward kernel
        if (it > 0) {
            if (it + 1 < n) issue(tgt, Jnext);
            Jnext = col_at(it + 2);
        }
        bf16x4 dsq[NKT];
#pragma unroll
        for (int kt = 0; kt < NKT; ++kt) {
            // dP - delta comes out of the MFMA: the accumulator starts at -delta instead of 0
            f32x4 s = f32x4{0.f, 0.f, 0.f, 0.f}, dp = f32x4{-delta, -delta, -delta, -delta};
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const int off = kt * 16 * kD + sl.frag[c];
                s = mma_d(s, *reinterpret_cast<const bf16x8*>(cur.k + off), qf[c]);      // S^T = K Q^T
                dp = mma_d(dp, *reinterpret_cast<const bf16x8*>(cur.v + off), dof[c]);   // dP^T = V dO^T
            }
            f32x4 ds;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float p = fast_exp2(fmaf(s[i], scale_log2, -lse2));
                ds[i] = p * dp[i];
            }
            dsq[kt] = to_quad<bf16_t>(ds);
        }
        mma_over_rows_swz<BS>(dq, cur.k, dsq, sl);    // dQ^T[d][query] += K^T dS^T
    };

    for (int it = 0; it < n; it += 2) {
        step(sm0, sm1, it);
        if (it + 1 < n) step(sm1, sm0, it + 1);
    }
    // an empty row never waited for its early load: it must land before this workgroup's LDS is freed
    __builtin_amdgcn_s_waitcnt(kWaitVm0);
    // through the stage the last block did not use (see the forward kernel)
    bf16_t* patch = ((n & 1) ? sm1.k : sm0.k) + wave * (16 * kD);
    store_rows_coalesced(patch, dQ + head + (size_t)(I * BS + wave * 16) * kD, dq, scale, lane);
}

// ------------------------------------------------------------------------------------------------
// backward, key side: one work item (a chunk of the kept rows of one block column) per workgroup.
// Three stages of {Q, dO, LSE, delta}: block it + 2 is loaded while block it is multiplied.  The
// accumulators of dK and dV cap the kernel at three workgroups per CU anyway, so the third stage is
// free.
// ------------------------------------------------------------------------------------------------
template <int BS>
struct DkvSmem {
    bf16_t q[BS * kD];
    bf16_t d[BS * kD];
    float lse[BS];
    float del[BS];
};

template <int BS>
__global__ __launch_bounds__(BS * 4) void attn_bwd_dkv_bf16_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const bf16_t* __restrict__ dO, const float* __restrict__ LSE2, const float* __restrict__ delta,
    bf16_t* __restrict__ dK, bf16_t* __restrict__ dV, const int* __restrict__ row_idx,
    const int4* __restrict__ sched, int w_max, int total, int n_slots, float* __restrict__ partial, int L,
    float scale, float scale_log2) {
    constexpr int NQT = BS / 16;
    // separate objects, so that the compiler can tell a read of one stage from a load in flight into
    // another and does not wait for it
    __shared__ __attribute__((aligned(16))) DkvSmem<BS> sm0, sm1, sm2;
    SPION_TP(0);

    // Work item w of head bh.  Each XCD works on whole heads (so a head's Q / dO stay in one L2), and
    // within an XCD the ids go item-major: the long items (low w) of all its heads are dispatched
    // before any short one, instead of one head's short items ahead of the next head's long ones.
    int w, bh;
    {
        const int BH = total / w_max;
        if ((BH & 7) == 0) {
            const int hpx = BH >> 3, x = blockIdx.x & 7, l = blockIdx.x >> 3;   // l-th workgroup of XCD x
            bh = x * hpx + l % hpx;
            w = l / hpx;
        } else {
            bh = blockIdx.x % BH;
            w = blockIdx.x / BH;
        }
    }
    const int4 item = sched[w], fr = sched[w_max + w];   // the item and its first four block rows
    const int J = item.x, n = item.z - item.y, slot = item.w;
    if (J < 0) return;
    const int tid = threadIdx.x, lane = tid & 63, r = lane & 15, g = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const size_t head = (size_t)bh * L * kD;
    const size_t vec = (size_t)bh * L;
    const int krow = J * BS + wave * 16 + r;
    const int last = n > 0 ? n - 1 : 0;
    const int* rows = row_idx + item.y;
    const SwzLane sl(r, g);
    const TileLoadLane tl(wave, lane);

    // a group of 4 tile loads per wave, plus one 4-byte-per-lane load in waves 0 (LSE) and 1 (delta)
    auto issue = [&](DkvSmem<BS>& st, int I) {
        tile_load_async(Q + head + (size_t)I * BS * kD, st.q, wave, tl);
        tile_load_async(dO + head + (size_t)I * BS * kD, st.d, wave, tl);
        if (wave == 0) {
            if (lane < BS)
                __builtin_amdgcn_global_load_lds(LSE2 + vec + (size_t)I * BS + lane, (lds_void_ptr)st.lse, 4, 0, 0);
        } else if (wave == 1) {
            if (lane < BS)
                __builtin_amdgcn_global_load_lds(delta + vec + (size_t)I * BS + lane, (lds_void_ptr)st.del, 4, 0, 0);
        }
    };

    int Ipre = fr.z;   // block of step it + 2
    if (n > 0) issue(sm0, fr.x);
    if (n > 1) issue(sm1, fr.y);
    // owned K / V fragments (step 0 waits for everything issued up to here)
    bf16x8 kf[2], vf[2];
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const size_t off = head + (size_t)krow * kD + c * 32 + g * 8;
        kf[c] = *reinterpret_cast<const bf16x8*>(K + off);
        vf[c] = *reinterpret_cast<const bf16x8*>(V + off);
    }

    f32x4 dk[4], dv[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
        dk[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
        dv[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    SPION_TP(1);
    auto step = [&](const DkvSmem<BS>& cur, DkvSmem<BS>& nxt2, int it) {
        if (it < 6) SPION_TP(2 + 2 * it);
        // wait until this wave's part of block `it` has landed; the group of block it + 1 may fly on
        if (it + 1 < n && it > 0) {
            if (wave < 2) __builtin_amdgcn_s_waitcnt(kWaitVm5);
            else __builtin_amdgcn_s_waitcnt(kWaitVm4);
        } else {
            __builtin_amdgcn_s_waitcnt(kWaitVm0);   // step 0 also waits for the owned K / V fragments
        }
        // everyone's part has landed and the stage of block it - 1 is no longer read.  A bare barrier:
        // the fences of __syncthreads would wait for every load in flight, the next block's included
        __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if (it < 6) SPION_TP(3 + 2 * it);
        if (it + 2 < n) issue(nxt2, Ipre);
        Ipre = it == 0 ? fr.w : rows[it + 3 < last ? it + 3 : last];
        bf16x4 pq[NQT], dsq[NQT];
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt) {
            // the query side stored -delta: as the initial accumulator it makes the MFMA return dP - delta
            f32x4 s = f32x4{0.f, 0.f, 0.f, 0.f};
            f32x4 dp = *reinterpret_cast<const f32x4*>(&cur.del[qt * 16 + 4 * g]);
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                s = mma_d(s, *reinterpret_cast<const bf16x8*>(cur.q + qt * 16 * kD + sl.frag[c]), kf[c]);    // S = Q K^T
                dp = mma_d(dp, *reinterpret_cast<const bf16x8*>(cur.d + qt * 16 * kD + sl.frag[c]), vf[c]);  // dP = dO V^T
            }
            const f32x4 lse4 = *reinterpret_cast<const f32x4*>(&cur.lse[qt * 16 + 4 * g]);   // log2 units
            f32x4 p, ds;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                p[i] = fast_exp2(fmaf(s[i], scale_log2, -lse4[i]));
                ds[i] = p[i] * dp[i];
            }
            pq[qt] = to_quad<bf16_t>(p);
            dsq[qt] = to_quad<bf16_t>(ds);
        }
        mma_over_rows_swz<BS>(dv, cur.d, pq, sl);    // dV^T[d][key] += dO^T P
        mma_over_rows_swz<BS>(dk, cur.q, dsq, sl);   // dK^T[d][key] += Q^T dS
    };

    for (int it = 0; it < n; it += 3) {
        step(sm0, sm2, it);
        if (it + 1 < n) step(sm1, sm0, it + 1);
        if (it + 2 < n) step(sm2, sm1, it + 2);
    }

    SPION_TP(14);
    if (slot < 0) {
        // stage n % 3 is free: its last reader was block n - 3, no load targets it any more, and the
        // only loads that ever touched this wave's 2 KB of its Q and dO tiles were the wave's own
        DkvSmem<BS>& fs = n % 3 == 0 ? sm0 : (n % 3 == 1 ? sm1 : sm2);
        const size_t row0 = head + (size_t)(J * BS + wave * 16) * kD;
        store_rows_coalesced(fs.q + wave * (16 * kD), dK + row0, dk, scale, lane);
        store_rows_coalesced(fs.d + wave * (16 * kD), dV + row0, dv, 1.f, lane);
    } else {
        // fp32 partial tile of this chunk, unscaled: [head][slot][dK | dV][bs][64]
        float* pk = partial + ((size_t)bh * n_slots + slot) * (2 * BS * kD) + (size_t)(wave * 16 + r) * kD;
        float* pv = pk + BS * kD;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
            *reinterpret_cast<f32x4*>(pk + dt * 16 + 4 * g) = dk[dt];
            *reinterpret_cast<f32x4*>(pv + dt * 16 + 4 * g) = dv[dt];
        }
    }
    SPION_TP(15);
}


// ------------------------------------------------------------------------------------------------
// launchers (called by the dispatch in attn_kernels.hip)
// ------------------------------------------------------------------------------------------------
template <int BS>
hipError_t fwd_bf16(const AttnShape& s, const void* Q, const void* K, const void* V, void* O, float* LSE,
                    const int* row_ptr, const int* col_idx, hipStream_t st) {
    const int total = s.nb * s.BH;
    attn_fwd_bf16_kernel<BS><<<dim3((unsigned)total), dim3(BS * 4), 0, st>>>(
        static_cast<const bf16_t*>(Q), static_cast<const bf16_t*>(K), static_cast<const bf16_t*>(V),
        static_cast<bf16_t*>(O), LSE, row_ptr, col_idx, s.L, s.nb, total, s.scale * kLog2e, s.paper_denom);
    return hipGetLastError();
}

template <int BS>
hipError_t bwd_dq_bf16(const AttnShape& s, const void* Q, const void* K, const void* V, const void* O,
                       const void* dO, const float* LSE, void* dQ, float* delta, float* lse2, const int* row_ptr,
                       const int* col_idx, const int* col_ptr, const int* row_idx, int w_max, int split_max,
                       int4* sched, int4* split, hipStream_t st) {
    const int total = s.nb * s.BH;
    attn_bwd_dq_bf16_kernel<BS><<<dim3((unsigned)total), dim3(BS * 4), 0, st>>>(
        static_cast<const bf16_t*>(Q), static_cast<const bf16_t*>(K), static_cast<const bf16_t*>(V),
        static_cast<const bf16_t*>(O), static_cast<const bf16_t*>(dO), LSE, static_cast<bf16_t*>(dQ), delta, lse2,
        row_ptr, col_idx, col_ptr, row_idx, w_max, split_max, sched, split, s.L, s.nb, total, s.scale,
        s.scale * kLog2e);
    return hipGetLastError();
}

template <int BS>
hipError_t bwd_dkv_bf16(const AttnShape& s, const void* Q, const void* K, const void* V, const void* dO,
                        const float* lse2, const float* delta, void* dK, void* dV, const int* row_idx,
                        const int4* sched, int w_max, int n_slots, float* partial, hipStream_t st) {
    const int total = w_max * s.BH;
    attn_bwd_dkv_bf16_kernel<BS><<<dim3((unsigned)total), dim3(BS * 4), 0, st>>>(
        static_cast<const bf16_t*>(Q), static_cast<const bf16_t*>(K), static_cast<const bf16_t*>(V),
        static_cast<const bf16_t*>(dO), lse2, delta, static_cast<bf16_t*>(dK), static_cast<bf16_t*>(dV),
        row_idx, sched, w_max, total, n_slots, partial, s.L, s.scale, s.scale * kLog2e);
    return hipGetLastError();
}

template hipError_t fwd_bf16<32>(const AttnShape&, const void*, const void*, const void*, void*, float*,
                                 const int*, const int*, hipStream_t);
template hipError_t fwd_bf16<64>(const AttnShape&, const void*, const void*, const void*, void*, float*,
                                 const int*, const int*, hipStream_t);
template hipError_t bwd_dq_bf16<32>(const AttnShape&, const void*, const void*, const void*, const void*,
                                    const void*, const float*, void*, float*, float*, const int*, const int*,
                                    const int*, const int*, int, int, int4*, int4*, hipStream_t);
template hipError_t bwd_dq_bf16<64>(const AttnShape&, const void*, const void*, const void*, const void*,
                                    const void*, const float*, void*, float*, float*, const int*, const int*,
                                    const int*, const int*, int, int, int4*, int4*, hipStream_t);
template hipError_t bwd_dkv_bf16<32>(const AttnShape&, const void*, const void*, const void*, const void*,
                                     const float*, const float*, void*, void*, const int*, const int4*,
                                     int, int, float*, hipStream_t);
template hipError_t bwd_dkv_bf16<64>(const AttnShape&, const void*, const void*, const void*, const void*,
                                     const float*, const float*, void*, void*, const int*, const int4*,
                                     int, int, float*, hipStream_t);

}  // namespace spion
