// bf16 block-sparse attention forward (Eq. 5 / Algorithm 5 lines 5-7, softmax as in Algorithm 6) tuned
// for gfx950, block size 32 or 64.
//
// Same mathematics and wave tiling as the generic kernels (16 owned rows per wave on the N index of
// every MFMA tile), plus:
//   - K / V tiles travel HBM -> LDS through the memory pipeline, one block ahead of the block being
//     multiplied, one barrier per kept block;
//   - the kernel starts loading the diagonal block before it has read the index;
//   - workgroup ids are remapped so that each of the 8 XCDs (one L2 each) works on whole heads.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "attn_bf16_tiles.h"
#include "attn_common.h"
#include "spion_internal.h"

namespace spion {

// ------------------------------------------------------------------------------------------------
// K / V tiles in two LDS stages, the next block loading while the
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

template <int BS>
__global__ __launch_bounds__(BS * 4) void attn_fwd_bf16_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    bf16_t* __restrict__ O, float* __restrict__ LSE, const int* __restrict__ row_ptr,
    const int* __restrict__ col_idx, int L, int nb, int total, float scale_log2, int paper_denom) {
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
        // loads in flight here: block `it`, and at step 0 also block 1, requested by the prologue (the
        // four youngest loads: whatever else the prologue stored or loaded after them only adds waiting)
        stage_ready(it == 0);
        if (it > 0) {
            if (it + 1 < n) issue(tgt, Jnext);
            Jnext = col_at(it + 2);
        }
        // S^T tile kt: [key 16 kt + 4 g + i][query r]; all K fragments are requested up front
        bf16x8 kfr[NKT][2];
#pragma unroll
        for (int kt = 0; kt < NKT; ++kt)
#pragma unroll
            for (int c = 0; c < 2; ++c)
                kfr[kt][c] = *reinterpret_cast<const bf16x8*>(cur.k + kt * 16 * kD + sl.frag[c]);
        f32x4 s[NKT];
        float mx = -INFINITY;
#pragma unroll
        for (int kt = 0; kt < NKT; ++kt) {
            s[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int c = 0; c < 2; ++c) s[kt] = mma_d(s[kt], kfr[kt][c], qf[c]);
        }
        // the transposed V operands of O^T += V^T P^T do not depend on P: requested here, they land
        // while the maxima and exponentials below are computed
        constexpr int NM = (BS / 32) * 4;
        bf16x8 vop[NM];
#pragma unroll
        for (int j = 0; j < NM; ++j) {
            const int o = sl.tr(j & 3) + (j >> 2) * 32 * kD;
            vop[j] = join(lds_read_tr(cur.v + o), lds_read_tr(cur.v + 16 * kD + o));
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kt = 0; kt < NKT; ++kt)
#pragma unroll
            for (int i = 0; i < 4; ++i) mx = fmaxf(mx, s[kt][i]);
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
#pragma unroll
        for (int j = 0; j < NM; ++j) {
            const int pc = j >> 2;
            oacc[j & 3] = mma_d(oacc[j & 3], vop[j], join(pq[2 * pc], pq[2 * pc + 1]));   // O^T[d][query] += V^T P^T
        }
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
    // the stage that the last block did not use is free: every wave is past the barrier that followed
    // its last reader, and the only load that ever targets this wave's 2 KB of it was the wave's own
    bf16_t* patch = ((n & 1) ? sm1.k : sm0.k) + wave * (16 * kD);
    store_rows_coalesced(patch, O + head + (size_t)(I * BS + wave * 16) * kD, oacc, inv, lane);
    if (g == 0) LSE[(size_t)bh * L + qrow] = lsum > 0.f ? (m + log2f(lsum)) * kLn2 : -INFINITY;
}

// ------------------------------------------------------------------------------------------------
// launcher (called by the dispatch in attn_kernels.hip)
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

template hipError_t fwd_bf16<32>(const AttnShape&, const void*, const void*, const void*, void*, float*,
                                 const int*, const int*, hipStream_t);
template hipError_t fwd_bf16<64>(const AttnShape&, const void*, const void*, const void*, void*, float*,
                                 const int*, const int*, hipStream_t);

}  // namespace spion
