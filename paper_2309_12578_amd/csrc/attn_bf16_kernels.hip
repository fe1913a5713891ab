// bf16 block-sparse attention kernels tuned for gfx950, block size 32 or 64.
//
// Same mathematics and wave tiling as the generic kernels (16 owned rows per wave on the N index of
// every MFMA tile), plus:
//   - tiles stay row-major in LDS; operands that must be read along the row index (V for O = P V,
//     K for dQ, Q and dO for dK / dV) come out of the same tile through the LDS transpose read
//     (ds_read_b64_tr_b16: 16 lanes fetch a 4 x 16 patch and each receives one column of it);
//   - LDS tiles are double buffered and the next tile travels HBM -> registers while the current one
//     is multiplied, so a kept block costs one barrier and no exposed memory round trip;
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

// LDS row stride in bf16 elements: 160 B.  Measured with SQ_LDS_BANK_CONFLICT: a 144 B stride costs
// 38-42 % extra LDS cycles (the transpose reads fetch 32 B from each of 8 consecutive rows, which
// tile the 64 banks only if the stride is an odd multiple of 32 B); 160 B has no conflicts for the
// 16-byte fragment reads, the transpose reads and the staging writes alike.
constexpr int kLd = kD + 16;

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

// One bs x 64 bf16 tile = bs * 8 fragments of 16 B; a workgroup of 4 * bs threads moves 2 each.
template <int BS>
struct TileRegs {
    bf16x8 f[2];
    __device__ __forceinline__ void load(const bf16_t* __restrict__ src, int tid) {
#pragma unroll
        for (int it = 0; it < 2; ++it)
            f[it] = *reinterpret_cast<const bf16x8*>(src + (size_t)(it * BS * 4 + tid) * 8);
    }
    __device__ __forceinline__ void store(bf16_t* lds, int tid) const {
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int idx = it * BS * 4 + tid;
            *reinterpret_cast<bf16x8*>(lds + (idx >> 3) * kLd + (idx & 7) * 8) = f[it];
        }
    }
};

// acc[dt][i] (d = 16 dt + 4 g + i, owned row r) += sum over the tile's rows of
// tile[row][16 dt + ...] * x[row][r], with x given as accumulator-layout tiles of 16 rows.
template <int BS>
__device__ __forceinline__ void mma_over_rows_tr(f32x4 (&acc)[4], const bf16_t* tile,
                                                 const bf16x4 (&x)[BS / 16], int r, int g) {
    const bf16_t* base = tile + (4 * g + (r >> 2)) * kLd + 4 * (r & 3);
#pragma unroll
    for (int pc = 0; pc < BS / 32; ++pc) {
        const bf16x8 xf = join(x[2 * pc], x[2 * pc + 1]);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
            const bf16x4 lo = lds_read_tr(base + (pc * 32) * kLd + dt * 16);
            const bf16x4 hi = lds_read_tr(base + (pc * 32 + 16) * kLd + dt * 16);
            acc[dt] = mma_d(acc[dt], join(lo, hi), xf);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// LDS budget and pipeline.  A workgroup may use at most ~32 KB of LDS if four are to share a CU
// (more than that and only three fit, which turns a one-round launch into two).  Of the two tiles a
// step needs, the one that is read until the end of the step is double buffered and the one that is
// only needed early is single buffered and refilled behind a mid-step barrier, while the MFMAs of the
// second half run: 3 tiles of 10 KB.  Tile it+1 waits in registers during step it; its loads were
// issued one step earlier, the block index it needs two steps earlier.
// ------------------------------------------------------------------------------------------------

// ------------------------------------------------------------------------------------------------
// forward
// ------------------------------------------------------------------------------------------------
template <int BS>
__global__ __launch_bounds__(BS * 4) void attn_fwd_bf16_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    bf16_t* __restrict__ O, float* __restrict__ LSE, const int* __restrict__ row_ptr,
    const int* __restrict__ col_idx, int L, int nb, int total, float scale_log2, int paper_denom) {
    constexpr int NKT = BS / 16;
    __shared__ __attribute__((aligned(16))) bf16_t k_s[2][BS * kLd];
    __shared__ __attribute__((aligned(16))) bf16_t v_s[BS * kLd];
    SPION_TP(0);

    const int vid = xcd_remap(blockIdx.x, total);
    const int I = vid % nb, bh = vid / nb;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r = lane & 15, g = lane >> 4;
    const size_t head = (size_t)bh * L * kD;
    const int qrow = I * BS + wave * 16 + r;
    const int jb = row_ptr[I], n = row_ptr[I + 1] - jb;
    const int last = n > 0 ? n - 1 : 0;
    const int* cols = col_idx + jb;
    // clamped reads stay inside this row's entries; an empty row reads nothing
    const int J0 = n > 0 ? cols[0] : 0, J1 = n > 0 ? cols[1 < last ? 1 : last] : 0;
    int Jpre = n > 0 ? cols[2 < last ? 2 : last] : 0;   // block index of tile it + 2

    TileRegs<BS> kreg, vreg;
    {
        TileRegs<BS> k0, v0;
        if (n > 0) {
            k0.load(K + head + (size_t)J0 * BS * kD, tid);
            v0.load(V + head + (size_t)J0 * BS * kD, tid);
        }
        if (n > 1) {
            kreg.load(K + head + (size_t)J1 * BS * kD, tid);
            vreg.load(V + head + (size_t)J1 * BS * kD, tid);
        }
        if (n > 0) {
            k0.store(k_s[0], tid);
            v0.store(v_s, tid);
        }
    }
    bf16x8 qf[2];
#pragma unroll
    for (int c = 0; c < 2; ++c)
        qf[c] = *reinterpret_cast<const bf16x8*>(Q + head + (size_t)qrow * kD + c * 32 + g * 8);
    __syncthreads();
    SPION_TP(1);

    float m = -INFINITY;   // running row maximum in log2 units (score * scale * log2 e)
    f32x4 lacc = f32x4{0.f, 0.f, 0.f, 0.f};   // running row sum, replicated in its 4 elements
    f32x4 oacc[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) oacc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    bf16x8 ones;
#pragma unroll
    for (int e = 0; e < 8; ++e) ones[e] = (bf16_t)1.0f;

    for (int it = 0; it < n; ++it) {
        const int buf = it & 1;
        const bool more = it + 1 < n, more2 = it + 2 < n;
        const size_t t2 = head + (size_t)Jpre * BS * kD;
        if (more) kreg.store(k_s[buf ^ 1], tid);
        if (more2) kreg.load(K + t2, tid);
        const bf16_t* kt_s = k_s[buf];
        // S^T tile kt: [key 16 kt + 4 g + i][query r]
        f32x4 s[NKT];
        float mx = -INFINITY;
#pragma unroll
        for (int kt = 0; kt < NKT; ++kt) {
            s[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const bf16x8 kf = *reinterpret_cast<const bf16x8*>(kt_s + (kt * 16 + r) * kLd + c * 32 + g * 8);
                s[kt] = mma_d(s[kt], kf, qf[c]);
            }
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
        if (it > 0) __syncthreads();                  // V tile of this step is in place
        mma_over_rows_tr<BS>(oacc, v_s, pq, r, g);    // O^T[d][query] += V^T P^T
        __syncthreads();                              // every wave is done with v_s and k_s[buf]
        if (more) vreg.store(v_s, tid);
        if (more2) vreg.load(V + t2, tid);
        Jpre = cols[it + 3 < last ? it + 3 : last];
        if (it < 12) SPION_TP(2 + it);
    }

    float lsum = lacc[0];
    if (paper_denom) {
        // Algorithm 6: every masked entry of the row counts as a score of 0
        const float masked = (float)(L - n * BS);
        const float mp = fmaxf(m, 0.f);
        const float a = exp2f(m - mp);
        lsum = lsum * a + masked * exp2f(-mp);
        m = mp;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) oacc[dt] *= a;
    }
    const float inv = lsum > 0.f ? 1.f / lsum : 0.f;
    bf16_t* orow = O + head + (size_t)qrow * kD;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) store_quad<bf16_t>(orow + dt * 16 + 4 * g, oacc[dt] * inv);
    if (g == 0) LSE[(size_t)bh * L + qrow] = lsum > 0.f ? (m + log2f(lsum)) * kLn2 : -INFINITY;
    SPION_TP(15);
}

// ------------------------------------------------------------------------------------------------
// backward, query side: delta = rowsum(dO .* O), dQ; also builds the key-side work list
// ------------------------------------------------------------------------------------------------
template <int BS>
__global__ __launch_bounds__(BS * 4) void attn_bwd_dq_bf16_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const bf16_t* __restrict__ O, const bf16_t* __restrict__ dO, const float* __restrict__ LSE,
    bf16_t* __restrict__ dQ, float* __restrict__ delta_out, const int* __restrict__ row_ptr,
    const int* __restrict__ col_idx, const int* __restrict__ col_ptr, int w_max, int split_max,
    int4* __restrict__ sched, int4* __restrict__ split, int L, int nb, int total, float scale,
    float scale_log2) {
    constexpr int NKT = BS / 16;
    __shared__ __attribute__((aligned(16))) bf16_t k_s[2][BS * kLd];
    __shared__ __attribute__((aligned(16))) bf16_t v_s[BS * kLd];
    SPION_TP(0);

    const int vid = xcd_remap(blockIdx.x, total);
    const int I = vid % nb, bh = vid / nb;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r = lane & 15, g = lane >> 4;
    const size_t head = (size_t)bh * L * kD;
    const int qrow = I * BS + wave * 16 + r;
    const int jb = row_ptr[I], n = row_ptr[I + 1] - jb;
    const int last = n > 0 ? n - 1 : 0;
    const int* cols = col_idx + jb;
    // clamped reads stay inside this row's entries; an empty row reads nothing
    const int J0 = n > 0 ? cols[0] : 0, J1 = n > 0 ? cols[1 < last ? 1 : last] : 0;
    int Jpre = n > 0 ? cols[2 < last ? 2 : last] : 0;

    TileRegs<BS> kreg, vreg;
    {
        TileRegs<BS> k0, v0;
        if (n > 0) {
            k0.load(K + head + (size_t)J0 * BS * kD, tid);
            v0.load(V + head + (size_t)J0 * BS * kD, tid);
        }
        if (n > 1) {
            kreg.load(K + head + (size_t)J1 * BS * kD, tid);
            vreg.load(V + head + (size_t)J1 * BS * kD, tid);
        }
        if (n > 0) {
            k0.store(k_s[0], tid);
            v0.store(v_s, tid);
        }
    }
    if (vid == 0 && tid < 64) build_key_schedule(col_ptr, nb, w_max, split_max, sched, split, tid);

    bf16x8 qf[2], dof[2];
    float delta = 0.f;
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const size_t off = head + (size_t)qrow * kD + c * 32 + g * 8;
        qf[c] = *reinterpret_cast<const bf16x8*>(Q + off);
        dof[c] = *reinterpret_cast<const bf16x8*>(dO + off);
        const bf16x8 of = *reinterpret_cast<const bf16x8*>(O + off);
#pragma unroll
        for (int e = 0; e < 8; ++e) delta = fmaf((float)dof[c][e], (float)of[e], delta);
    }
    delta = group_sum(delta);
    if (g == 0) delta_out[(size_t)bh * L + qrow] = delta;
    const float lse2 = LSE[(size_t)bh * L + qrow] * kLog2e;
    __syncthreads();

    f32x4 dq[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) dq[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int it = 0; it < n; ++it) {
        const int buf = it & 1;
        const bool more = it + 1 < n, more2 = it + 2 < n;
        const size_t t2 = head + (size_t)Jpre * BS * kD;
        if (more) kreg.store(k_s[buf ^ 1], tid);
        if (more2) kreg.load(K + t2, tid);
        bf16x4 dsq[NKT];
#pragma unroll
        for (int kt = 0; kt < NKT; ++kt) {
            f32x4 s = f32x4{0.f, 0.f, 0.f, 0.f}, dp = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const int off = (kt * 16 + r) * kLd + c * 32 + g * 8;
                s = mma_d(s, *reinterpret_cast<const bf16x8*>(k_s[buf] + off), qf[c]);   // S^T = K Q^T
                dp = mma_d(dp, *reinterpret_cast<const bf16x8*>(v_s + off), dof[c]);     // dP^T = V dO^T
            }
            f32x4 ds;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float p = fast_exp2(fmaf(s[i], scale_log2, -lse2));
                ds[i] = p * (dp[i] - delta);
            }
            dsq[kt] = to_quad<bf16_t>(ds);
        }
        __syncthreads();                                  // every wave is done with v_s
        if (more) vreg.store(v_s, tid);
        if (more2) vreg.load(V + t2, tid);
        mma_over_rows_tr<BS>(dq, k_s[buf], dsq, r, g);    // dQ^T[d][query] += K^T dS^T
        Jpre = cols[it + 3 < last ? it + 3 : last];
        __syncthreads();                                  // k_s[buf] free, next V and K tiles in place
    }
    bf16_t* drow = dQ + head + (size_t)qrow * kD;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) store_quad<bf16_t>(drow + dt * 16 + 4 * g, dq[dt] * scale);
}

// ------------------------------------------------------------------------------------------------
// backward, key side: one work item (a chunk of the kept rows of one block column) per workgroup
// ------------------------------------------------------------------------------------------------
template <int BS>
__global__ __launch_bounds__(BS * 4) void attn_bwd_dkv_bf16_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const bf16_t* __restrict__ dO, const float* __restrict__ LSE, const float* __restrict__ delta,
    bf16_t* __restrict__ dK, bf16_t* __restrict__ dV, const int* __restrict__ row_idx,
    const int4* __restrict__ sched, int w_max, int total, int n_slots, float* __restrict__ partial, int L,
    float scale, float scale_log2) {
    constexpr int NQT = BS / 16;
    __shared__ __attribute__((aligned(16))) bf16_t q_s[2][BS * kLd];
    __shared__ __attribute__((aligned(16))) bf16_t do_s[BS * kLd];
    __shared__ __attribute__((aligned(16))) float lse_s[2][BS];
    __shared__ __attribute__((aligned(16))) float delta_s[2][BS];

    const int vid = xcd_remap(blockIdx.x, total);
    const int w = vid % w_max, bh = vid / w_max;
    const int4 item = sched[w];
    const int J = item.x, n = item.z - item.y, slot = item.w;
    if (J < 0) return;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r = lane & 15, g = lane >> 4;
    const size_t head = (size_t)bh * L * kD;
    const size_t vec = (size_t)bh * L;
    const int krow = J * BS + wave * 16 + r;
    const int last = n > 0 ? n - 1 : 0;
    const int* rows = row_idx + item.y;
    const int I0 = n > 0 ? rows[0] : 0, I1 = n > 0 ? rows[1 < last ? 1 : last] : 0;
    int Ipre = n > 0 ? rows[2 < last ? 2 : last] : 0;

    TileRegs<BS> qreg, doreg;
    float lse_r = 0.f, delta_r = 0.f;
    {
        TileRegs<BS> q0, do0;
        float lse0 = 0.f, delta0 = 0.f;
        if (n > 0) {
            q0.load(Q + head + (size_t)I0 * BS * kD, tid);
            do0.load(dO + head + (size_t)I0 * BS * kD, tid);
            if (tid < BS) {
                lse0 = LSE[vec + I0 * BS + tid];
                delta0 = delta[vec + I0 * BS + tid];
            }
        }
        if (n > 1) {
            qreg.load(Q + head + (size_t)I1 * BS * kD, tid);
            doreg.load(dO + head + (size_t)I1 * BS * kD, tid);
            if (tid < BS) {
                lse_r = LSE[vec + I1 * BS + tid];
                delta_r = delta[vec + I1 * BS + tid];
            }
        }
        if (n > 0) {
            q0.store(q_s[0], tid);
            do0.store(do_s, tid);
            if (tid < BS) {
                lse_s[0][tid] = lse0 * kLog2e;
                delta_s[0][tid] = delta0;
            }
        }
    }
    bf16x8 kf[2], vf[2];
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const size_t off = head + (size_t)krow * kD + c * 32 + g * 8;
        kf[c] = *reinterpret_cast<const bf16x8*>(K + off);
        vf[c] = *reinterpret_cast<const bf16x8*>(V + off);
    }
    __syncthreads();

    f32x4 dk[4], dv[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
        dk[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
        dv[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    for (int it = 0; it < n; ++it) {
        const int buf = it & 1;
        const bool more = it + 1 < n, more2 = it + 2 < n;
        const size_t t2 = head + (size_t)Ipre * BS * kD;
        const size_t v2 = vec + (size_t)Ipre * BS + tid;
        if (more) {
            qreg.store(q_s[buf ^ 1], tid);
            if (tid < BS) {
                lse_s[buf ^ 1][tid] = lse_r * kLog2e;
                delta_s[buf ^ 1][tid] = delta_r;
            }
        }
        if (more2) {
            qreg.load(Q + t2, tid);
            if (tid < BS) {
                lse_r = LSE[v2];
                delta_r = delta[v2];
            }
        }
        bf16x4 pq[NQT], dsq[NQT];
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt) {
            f32x4 s = f32x4{0.f, 0.f, 0.f, 0.f}, dp = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const int off = (qt * 16 + r) * kLd + c * 32 + g * 8;
                s = mma_d(s, *reinterpret_cast<const bf16x8*>(q_s[buf] + off), kf[c]);   // S = Q K^T
                dp = mma_d(dp, *reinterpret_cast<const bf16x8*>(do_s + off), vf[c]);     // dP = dO V^T
            }
            const f32x4 lse4 = *reinterpret_cast<const f32x4*>(&lse_s[buf][qt * 16 + 4 * g]);
            const f32x4 del4 = *reinterpret_cast<const f32x4*>(&delta_s[buf][qt * 16 + 4 * g]);
            f32x4 p, ds;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                p[i] = fast_exp2(fmaf(s[i], scale_log2, -lse4[i]));
                ds[i] = p[i] * (dp[i] - del4[i]);
            }
            pq[qt] = to_quad<bf16_t>(p);
            dsq[qt] = to_quad<bf16_t>(ds);
        }
        mma_over_rows_tr<BS>(dv, do_s, pq, r, g);          // dV^T[d][key] += dO^T P
        __syncthreads();                                    // every wave is done with do_s
        if (more) doreg.store(do_s, tid);
        if (more2) doreg.load(dO + t2, tid);
        mma_over_rows_tr<BS>(dk, q_s[buf], dsq, r, g);      // dK^T[d][key] += Q^T dS
        Ipre = rows[it + 3 < last ? it + 3 : last];
        __syncthreads();                                    // q_s[buf] free, next tiles in place
    }
    if (slot < 0) {
        bf16_t* dkrow = dK + head + (size_t)krow * kD;
        bf16_t* dvrow = dV + head + (size_t)krow * kD;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
            store_quad<bf16_t>(dkrow + dt * 16 + 4 * g, dk[dt] * scale);
            store_quad<bf16_t>(dvrow + dt * 16 + 4 * g, dv[dt]);
        }
    } else {
        // fp32 partial tile of this chunk, unscaled: [head][slot][dK | dV][bs][64]; a second kernel
        // adds the chunks of a column in chunk order (a kernel boundary is the cheapest way to make
        // the tiles visible across XCDs: a device-scope release inside the kernel flushes the whole L2)
        float* pk = partial + ((size_t)bh * n_slots + slot) * (2 * BS * kD) + (size_t)(wave * 16 + r) * kD;
        float* pv = pk + BS * kD;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
            *reinterpret_cast<f32x4*>(pk + dt * 16 + 4 * g) = dk[dt];
            *reinterpret_cast<f32x4*>(pv + dt * 16 + 4 * g) = dv[dt];
        }
    }
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
                       const void* dO, const float* LSE, void* dQ, float* delta, const int* row_ptr,
                       const int* col_idx, const int* col_ptr, int w_max, int split_max, int4* sched,
                       int4* split, hipStream_t st) {
    const int total = s.nb * s.BH;
    attn_bwd_dq_bf16_kernel<BS><<<dim3((unsigned)total), dim3(BS * 4), 0, st>>>(
        static_cast<const bf16_t*>(Q), static_cast<const bf16_t*>(K), static_cast<const bf16_t*>(V),
        static_cast<const bf16_t*>(O), static_cast<const bf16_t*>(dO), LSE, static_cast<bf16_t*>(dQ), delta,
        row_ptr, col_idx, col_ptr, w_max, split_max, sched, split, s.L, s.nb, total, s.scale,
        s.scale * kLog2e);
    return hipGetLastError();
}

template <int BS>
hipError_t bwd_dkv_bf16(const AttnShape& s, const void* Q, const void* K, const void* V, const void* dO,
                        const float* LSE, const float* delta, void* dK, void* dV, const int* row_idx,
                        const int4* sched, int w_max, int n_slots, float* partial, hipStream_t st) {
    const int total = w_max * s.BH;
    attn_bwd_dkv_bf16_kernel<BS><<<dim3((unsigned)total), dim3(BS * 4), 0, st>>>(
        static_cast<const bf16_t*>(Q), static_cast<const bf16_t*>(K), static_cast<const bf16_t*>(V),
        static_cast<const bf16_t*>(dO), LSE, delta, static_cast<bf16_t*>(dK), static_cast<bf16_t*>(dV),
        row_idx, sched, w_max, total, n_slots, partial, s.L, s.scale, s.scale * kLog2e);
    return hipGetLastError();
}

template hipError_t fwd_bf16<32>(const AttnShape&, const void*, const void*, const void*, void*, float*,
                                 const int*, const int*, hipStream_t);
template hipError_t fwd_bf16<64>(const AttnShape&, const void*, const void*, const void*, void*, float*,
                                 const int*, const int*, hipStream_t);
template hipError_t bwd_dq_bf16<32>(const AttnShape&, const void*, const void*, const void*, const void*,
                                    const void*, const float*, void*, float*, const int*, const int*,
                                    const int*, int, int, int4*, int4*, hipStream_t);
template hipError_t bwd_dq_bf16<64>(const AttnShape&, const void*, const void*, const void*, const void*,
                                    const void*, const float*, void*, float*, const int*, const int*,
                                    const int*, int, int, int4*, int4*, hipStream_t);
template hipError_t bwd_dkv_bf16<32>(const AttnShape&, const void*, const void*, const void*, const void*,
                                     const float*, const float*, void*, void*, const int*, const int4*,
                                     int, int, float*, hipStream_t);
template hipError_t bwd_dkv_bf16<64>(const AttnShape&, const void*, const void*, const void*, const void*,
                                     const float*, const float*, void*, void*, const int*, const int4*,
                                     int, int, float*, hipStream_t);

}  // namespace spion
