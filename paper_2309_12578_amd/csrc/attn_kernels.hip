// Block-sparse attention forward and backward for gfx950 (Eq. 5 / Algorithm 5 lines 4-7 of the SPION
// paper, softmax as in Algorithm 6, gradient by the chain rule).
//
// One pattern (BSR, plus BSC for the backward) is shared by all batch items and heads.  A kept block
// is a dense bs x bs tile, so SDDMM and SpMM inside it are dense contractions and run on MFMA; the
// row softmax is fused between them and never touches HBM.
//
// Wave-level tiling (wave64).  A wave owns 16 rows (queries in the row-walking kernels, keys in the
// column-walking one) and all 64 head-dim columns.  Every product is issued so that the 16 owned
// rows sit on the N index of a 16x16 MFMA tile: lane l then holds values for owned row l % 16 only,
// which makes row statistics (max, sum, LSE, delta) lane-uniform scalars, and makes an fp32
// accumulator tile directly usable as the B operand of the next product (accumulator element i of
// lane group g = l / 16 is contraction index 4 g + i, the same lanes a B fragment needs).
//
// The other operand of a product that contracts over keys (or queries) must be read along that
// index; tiles are therefore staged in LDS twice where needed: row-major [row][d] for products that
// contract over d, and transposed [d][row] for products that contract over rows.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "attn_common.h"
#include "spion_internal.h"

namespace spion {

// ------------------------------------------------------------------------------------------------
// forward: workgroup = (head, block row I); wave w owns query rows I*bs + 16 w .. + 15
// ------------------------------------------------------------------------------------------------
template <typename T, int BS>
__global__ __launch_bounds__(BS * 4) void attn_fwd_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V, T* __restrict__ O,
    float* __restrict__ LSE, const int* __restrict__ row_ptr, const int* __restrict__ col_idx, int L,
    int nb, float scale_log2, int paper_denom) {
    typedef typename Elem<T>::Frag Frag;
    typedef typename Elem<T>::Quad Quad;
    constexpr int EPL = Elem<T>::EPL, KC = Elem<T>::KC, NDC = kD / KC, NKT = BS / 16;
    constexpr int LDK = kD + EPL, LDT = BS + EPL;
    __shared__ __attribute__((aligned(16))) T k_rm[BS * LDK];
    __shared__ __attribute__((aligned(16))) T v_tr[kD * LDT];

    const int I = blockIdx.x % nb, bh = blockIdx.x / nb;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r = lane & 15, g = lane >> 4;
    const size_t head = (size_t)bh * L * kD;
    const int qrow = I * BS + wave * 16 + r;

    Frag qf[NDC];
#pragma unroll
    for (int c = 0; c < NDC; ++c)
        qf[c] = *reinterpret_cast<const Frag*>(Q + head + (size_t)qrow * kD + c * KC + g * EPL);

    float m = -INFINITY, lsum = 0.f;   // m in log2 units (score * scale * log2 e)
    f32x4 oacc[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) oacc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int jb = row_ptr[I], je = row_ptr[I + 1];
    for (int j = jb; j < je; ++j) {
        const int J = col_idx[j];
        __syncthreads();
        stage_tile<T, BS, LDK, LDT, true, false>(K + head + (size_t)J * BS * kD, k_rm, nullptr, tid);
        stage_tile<T, BS, LDK, LDT, false, true>(V + head + (size_t)J * BS * kD, nullptr, v_tr, tid);
        __syncthreads();

        // S^T tile kt: [key 16 kt + 4 g + i][query r]
        f32x4 s[NKT];
        float mx = -INFINITY;
#pragma unroll
        for (int kt = 0; kt < NKT; ++kt) {
            s[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int c = 0; c < NDC; ++c) {
                const Frag kf = *reinterpret_cast<const Frag*>(k_rm + (kt * 16 + r) * LDK + c * KC + g * EPL);
                s[kt] = mma_d(s[kt], kf, qf[c]);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) mx = fmaxf(mx, s[kt][i]);
        }
        mx = group_max(mx);
        const float m_new = fmaxf(m, mx * scale_log2);
        const float alpha = exp2f(m - m_new);
        lsum *= alpha;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) oacc[dt] *= alpha;
        Quad pq[NKT];
#pragma unroll
        for (int kt = 0; kt < NKT; ++kt) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float p = exp2f(fmaf(s[kt][i], scale_log2, -m_new));
                s[kt][i] = p;
                lsum += p;
            }
            pq[kt] = to_quad<T>(s[kt]);
        }
        m = m_new;
        mma_over_rows<T, BS, LDT>(oacc, v_tr, pq, r, g);   // O^T[d][query] += V^T P^T
    }

    lsum = group_sum(lsum);
    if (paper_denom && je > jb) {
        // Algorithm 6: every masked entry of the row counts as a score of 0 (a row that keeps nothing
        // has no entry to normalise and stays at O = 0, LSE = -inf)
        const float masked = (float)(L - (je - jb) * BS);
        const float mp = fmaxf(m, 0.f);
        const float a = exp2f(m - mp);
        lsum = lsum * a + masked * exp2f(-mp);
        m = mp;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) oacc[dt] *= a;
    }
    const float inv = lsum > 0.f ? 1.f / lsum : 0.f;
    T* orow = O + head + (size_t)qrow * kD;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) store_quad<T>(orow + dt * 16 + 4 * g, oacc[dt] * inv);
    if (g == 0) LSE[(size_t)bh * L + qrow] = lsum > 0.f ? (m + log2f(lsum)) * kLn2 : -INFINITY;
}

// ------------------------------------------------------------------------------------------------
// backward, query side: workgroup = (head, block row I).  Computes delta = rowsum(dO .* O) for its
// rows (stored for the key-side kernel) and dQ.
// ------------------------------------------------------------------------------------------------
template <typename T, int BS>
__global__ __launch_bounds__(BS * 4) void attn_bwd_dq_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V, const T* __restrict__ O,
    const T* __restrict__ dO, const float* __restrict__ LSE, T* __restrict__ dQ,
    float* __restrict__ delta_out, const int* __restrict__ row_ptr, const int* __restrict__ col_idx,
    const int* __restrict__ col_ptr, const int* __restrict__ row_idx, int w_max, int split_max,
    int4* __restrict__ sched, int4* __restrict__ split,
    int L, int nb, float scale, float scale_log2) {
    if (blockIdx.x == 0 && threadIdx.x < 64)
        build_key_schedule(col_ptr, row_idx, nb, w_max, split_max, sched, split, threadIdx.x);
    typedef typename Elem<T>::Frag Frag;
    typedef typename Elem<T>::Quad Quad;
    constexpr int EPL = Elem<T>::EPL, KC = Elem<T>::KC, NDC = kD / KC, NKT = BS / 16;
    constexpr int LDK = kD + EPL, LDT = BS + EPL;
    __shared__ __attribute__((aligned(16))) T k_rm[BS * LDK];
    __shared__ __attribute__((aligned(16))) T v_rm[BS * LDK];
    __shared__ __attribute__((aligned(16))) T k_tr[kD * LDT];

    const int I = blockIdx.x % nb, bh = blockIdx.x / nb;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r = lane & 15, g = lane >> 4;
    const size_t head = (size_t)bh * L * kD;
    const int qrow = I * BS + wave * 16 + r;

    Frag qf[NDC], dof[NDC];
    float delta = 0.f;
#pragma unroll
    for (int c = 0; c < NDC; ++c) {
        const size_t off = head + (size_t)qrow * kD + c * KC + g * EPL;
        qf[c] = *reinterpret_cast<const Frag*>(Q + off);
        dof[c] = *reinterpret_cast<const Frag*>(dO + off);
        const Frag of = *reinterpret_cast<const Frag*>(O + off);
#pragma unroll
        for (int e = 0; e < EPL; ++e) delta = fmaf((float)dof[c][e], (float)of[e], delta);
    }
    delta = group_sum(delta);
    if (g == 0) delta_out[(size_t)bh * L + qrow] = delta;
    const float lse2 = LSE[(size_t)bh * L + qrow] * kLog2e;

    f32x4 dq[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) dq[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int jb = row_ptr[I], je = row_ptr[I + 1];
    for (int j = jb; j < je; ++j) {
        const int J = col_idx[j];
        __syncthreads();
        stage_tile<T, BS, LDK, LDT, true, true>(K + head + (size_t)J * BS * kD, k_rm, k_tr, tid);
        stage_tile<T, BS, LDK, LDT, true, false>(V + head + (size_t)J * BS * kD, v_rm, nullptr, tid);
        __syncthreads();
        Quad dsq[NKT];
#pragma unroll
        for (int kt = 0; kt < NKT; ++kt) {
            f32x4 s = f32x4{0.f, 0.f, 0.f, 0.f}, dp = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int c = 0; c < NDC; ++c) {
                const int off = (kt * 16 + r) * LDK + c * KC + g * EPL;
                s = mma_d(s, *reinterpret_cast<const Frag*>(k_rm + off), qf[c]);     // S^T = K Q^T
                dp = mma_d(dp, *reinterpret_cast<const Frag*>(v_rm + off), dof[c]);  // dP^T = V dO^T
            }
            f32x4 ds;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float p = exp2f(fmaf(s[i], scale_log2, -lse2));
                ds[i] = p * (dp[i] - delta);
            }
            dsq[kt] = to_quad<T>(ds);
        }
        mma_over_rows<T, BS, LDT>(dq, k_tr, dsq, r, g);   // dQ^T[d][query] += K^T dS^T
    }
    T* drow = dQ + head + (size_t)qrow * kD;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) store_quad<T>(drow + dt * 16 + 4 * g, dq[dt] * scale);
}

// ------------------------------------------------------------------------------------------------
// backward, key side: workgroup = (head, work item w) with sched[w] = a chunk of the kept rows of
// block column J; wave w owns keys J*bs + 16 w .. + 15.  Deterministic: no atomics, one writer per
// output or per partial slot.
// ------------------------------------------------------------------------------------------------
template <typename T, int BS>
__global__ __launch_bounds__(BS * 4) void attn_bwd_dkv_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V, const T* __restrict__ dO,
    const float* __restrict__ LSE, const float* __restrict__ delta, T* __restrict__ dK,
    T* __restrict__ dV, const int* __restrict__ row_idx, const int4* __restrict__ sched, int w_max,
    int n_slots, float* __restrict__ partial, int L, float scale, float scale_log2) {
    typedef typename Elem<T>::Frag Frag;
    typedef typename Elem<T>::Quad Quad;
    constexpr int EPL = Elem<T>::EPL, KC = Elem<T>::KC, NDC = kD / KC, NQT = BS / 16;
    constexpr int LDK = kD + EPL, LDT = BS + EPL;
    __shared__ __attribute__((aligned(16))) T q_rm[BS * LDK];
    __shared__ __attribute__((aligned(16))) T do_rm[BS * LDK];
    __shared__ __attribute__((aligned(16))) T q_tr[kD * LDT];
    __shared__ __attribute__((aligned(16))) T do_tr[kD * LDT];
    __shared__ float lse_s[BS], delta_s[BS];

    const int w = blockIdx.x % w_max, bh = blockIdx.x / w_max;
    const int4 item = sched[w];
    const int J = item.x, kb = item.y, ke = item.z, slot = item.w;
    if (J < 0) return;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r = lane & 15, g = lane >> 4;
    const size_t head = (size_t)bh * L * kD;
    const int krow = J * BS + wave * 16 + r;

    Frag kf[NDC], vf[NDC];
#pragma unroll
    for (int c = 0; c < NDC; ++c) {
        const size_t off = head + (size_t)krow * kD + c * KC + g * EPL;
        kf[c] = *reinterpret_cast<const Frag*>(K + off);
        vf[c] = *reinterpret_cast<const Frag*>(V + off);
    }
    f32x4 dk[4], dv[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
        dk[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
        dv[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    for (int k = kb; k < ke; ++k) {
        const int I = row_idx[k];
        __syncthreads();
        stage_tile<T, BS, LDK, LDT, true, true>(Q + head + (size_t)I * BS * kD, q_rm, q_tr, tid);
        stage_tile<T, BS, LDK, LDT, true, true>(dO + head + (size_t)I * BS * kD, do_rm, do_tr, tid);
        if (tid < BS) {
            lse_s[tid] = LSE[(size_t)bh * L + I * BS + tid] * kLog2e;
            delta_s[tid] = delta[(size_t)bh * L + I * BS + tid];
        }
        __syncthreads();
        Quad pq[NQT], dsq[NQT];
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt) {
            f32x4 s = f32x4{0.f, 0.f, 0.f, 0.f}, dp = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int c = 0; c < NDC; ++c) {
                const int off = (qt * 16 + r) * LDK + c * KC + g * EPL;
                s = mma_d(s, *reinterpret_cast<const Frag*>(q_rm + off), kf[c]);     // S = Q K^T
                dp = mma_d(dp, *reinterpret_cast<const Frag*>(do_rm + off), vf[c]);  // dP = dO V^T
            }
            f32x4 p, ds;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int q = qt * 16 + 4 * g + i;
                p[i] = exp2f(fmaf(s[i], scale_log2, -lse_s[q]));
                ds[i] = p[i] * (dp[i] - delta_s[q]);
            }
            pq[qt] = to_quad<T>(p);
            dsq[qt] = to_quad<T>(ds);
        }
        mma_over_rows<T, BS, LDT>(dv, do_tr, pq, r, g);   // dV^T[d][key] += dO^T P
        mma_over_rows<T, BS, LDT>(dk, q_tr, dsq, r, g);   // dK^T[d][key] += Q^T dS
    }
    if (slot < 0) {
        T* dkrow = dK + head + (size_t)krow * kD;
        T* dvrow = dV + head + (size_t)krow * kD;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
            store_quad<T>(dkrow + dt * 16 + 4 * g, dk[dt] * scale);
            store_quad<T>(dvrow + dt * 16 + 4 * g, dv[dt]);
        }
    } else {
        // fp32 partial tiles [head][slot][dK | dV][bs][64], unscaled
        float* pk = partial + ((size_t)bh * n_slots + slot) * (2 * BS * kD) + (size_t)(wave * 16 + r) * kD;
        float* pv = pk + BS * kD;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
            *reinterpret_cast<f32x4*>(pk + dt * 16 + 4 * g) = dk[dt];
            *reinterpret_cast<f32x4*>(pv + dt * 16 + 4 * g) = dv[dt];
        }
    }
}

// Adds the partial tiles of every block column that was cut into several chunks, in chunk order.
// workgroup = (head, m-th split column, part): 256 threads, one float4 of the output tile each,
// bs / 16 parts per tile, so that the loads of all chunks of a float4 are in flight together.
template <typename T, int BS>
__global__ __launch_bounds__(256) void attn_bwd_dkv_reduce_kernel(
    const float* __restrict__ partial, const int4* __restrict__ split, int split_max, int n_slots,
    T* __restrict__ dK, T* __restrict__ dV, int L, float scale) {
    constexpr int PARTS = BS / 16;
    const int part = blockIdx.x % PARTS, m = (blockIdx.x / PARTS) % split_max;
    const int bh = blockIdx.x / (PARTS * split_max);
    const int4 info = split[m];   // {J, first slot, chunks}
    if (info.x < 0) return;
    const int v = part * 256 + threadIdx.x;
    const float* pk = partial + ((size_t)bh * n_slots + info.y) * (2 * BS * kD) + v * 4;
    f32x4 ak = f32x4{0.f, 0.f, 0.f, 0.f}, av = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
    for (int c = 0; c < info.z; ++c) {
        ak += *reinterpret_cast<const f32x4*>(pk + (size_t)c * (2 * BS * kD));
        av += *reinterpret_cast<const f32x4*>(pk + (size_t)c * (2 * BS * kD) + BS * kD);
    }
    const size_t out = (size_t)bh * L * kD + (size_t)info.x * BS * kD + v * 4;
    store_quad<T>(dK + out, ak * scale);
    store_quad<T>(dV + out, av);
}

// ------------------------------------------------------------------------------------------------
// host launchers
// ------------------------------------------------------------------------------------------------
size_t attn_bwd_workspace_bytes(int BH, int L, int bs, int nb, int nnzb) {
    const BwdWorkspace ws(BH, L, bs, nb, nnzb);
    return ws.total;
}

bool attn_bwd_grids_fit(int BH, int L, int bs, int nb, int nnzb) {
    const BwdWorkspace ws(BH, L, bs, nb, nnzb);
    const int64_t limit = 0x7fffffffll;
    return (int64_t)(ws.w_max + nb) * BH <= limit && (int64_t)ws.split_max * BH * (bs / 16) <= limit;
}

BwdWorkspace::BwdWorkspace(int BH, int L, int bs, int nb, int nnzb) {
    auto up = [](size_t x) { return (x + 255) / 256 * 256; };
    w_max = key_work_items_max(nnzb, nb);
    n_slots = key_slots_max(nnzb);
    delta_off = 0;
    sched_off = delta_off + up((size_t)2 * BH * L * sizeof(float));   // delta, then LSE in log2 units
    split_max = key_split_max(nnzb);
    split_off = sched_off + up((size_t)2 * w_max * sizeof(int4));   // items, then their first rows
    partial_off = split_off + up((size_t)split_max * sizeof(int4));
    total = partial_off + up((size_t)BH * n_slots * 2 * bs * kD * sizeof(float));
}

template <typename T, int BS>
static hipError_t fwd_t(const AttnShape& s, const void* Q, const void* K, const void* V, void* O,
                        float* LSE, const int* row_ptr, const int* col_idx, hipStream_t st) {
    if constexpr (sizeof(T) == 2 && BS >= 32) return fwd_bf16<BS>(s, Q, K, V, O, LSE, row_ptr, col_idx, st);
    attn_fwd_kernel<T, BS><<<dim3((unsigned)(s.nb * s.BH)), dim3(BS * 4), 0, st>>>(
        static_cast<const T*>(Q), static_cast<const T*>(K), static_cast<const T*>(V),
        static_cast<T*>(O), LSE, row_ptr, col_idx, s.L, s.nb, s.scale * kLog2e, s.paper_denom);
    return hipGetLastError();
}

template <typename T, int BS>
static hipError_t bwd_t(const AttnShape& s, const void* Q, const void* K, const void* V, const void* O,
                        const void* dO, const float* LSE, void* dQ, void* dK, void* dV,
                        const int* row_ptr, const int* col_idx, const int* col_ptr, const int* row_idx,
                        int nnzb, void* workspace, hipStream_t st) {
    const BwdWorkspace ws(s.BH, s.L, s.bs, s.nb, nnzb);
    char* base = static_cast<char*>(workspace);
    float* delta = reinterpret_cast<float*>(base + ws.delta_off);
    int4* sched = reinterpret_cast<int4*>(base + ws.sched_off);
    int4* split = reinterpret_cast<int4*>(base + ws.split_off);
    float* partial = reinterpret_cast<float*>(base + ws.partial_off);
    const dim3 block(BS * 4);
    if constexpr (sizeof(T) == 2 && BS >= 32) {
        // tuned bf16 path: one launch for both sides (it needs no delta, work list or split list in the
        // workspace), plus the small reduction of the partial tiles
        return bwd_bf16<BS>(s, Q, K, V, O, dO, LSE, dQ, dK, dV, row_ptr, col_idx, col_ptr, row_idx, nnzb, ws.w_max,
                            ws.split_max, ws.n_slots, partial, st);
    } else {
        if (s.bwd_phases & 1) {
            attn_bwd_dq_kernel<T, BS><<<dim3((unsigned)(s.nb * s.BH)), block, 0, st>>>(
                static_cast<const T*>(Q), static_cast<const T*>(K), static_cast<const T*>(V),
                static_cast<const T*>(O), static_cast<const T*>(dO), LSE, static_cast<T*>(dQ), delta,
                row_ptr, col_idx, col_ptr, row_idx, ws.w_max, ws.split_max, sched, split, s.L, s.nb, s.scale,
                s.scale * kLog2e);
            const hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
        if (s.bwd_phases & 2) {
            attn_bwd_dkv_kernel<T, BS><<<dim3((unsigned)(ws.w_max * s.BH)), block, 0, st>>>(
                static_cast<const T*>(Q), static_cast<const T*>(K), static_cast<const T*>(V),
                static_cast<const T*>(dO), LSE, delta, static_cast<T*>(dK), static_cast<T*>(dV), row_idx,
                sched, ws.w_max, ws.n_slots, partial, s.L, s.scale, s.scale * kLog2e);
            const hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
            attn_bwd_dkv_reduce_kernel<T, BS><<<dim3((unsigned)(ws.split_max * s.BH * (BS / 16))), dim3(256), 0, st>>>(
                partial, split, ws.split_max, ws.n_slots, static_cast<T*>(dK), static_cast<T*>(dV), s.L, s.scale);
        }
        return hipGetLastError();
    }
}

#define SPION_DISPATCH(FN, ...)                                                   \
    do {                                                                          \
        if (s.is_bf16) {                                                          \
            if (s.bs == 16) return FN<bf16_t, 16>(__VA_ARGS__);                   \
            if (s.bs == 32) return FN<bf16_t, 32>(__VA_ARGS__);                   \
            return FN<bf16_t, 64>(__VA_ARGS__);                                   \
        }                                                                         \
        if (s.bs == 16) return FN<float, 16>(__VA_ARGS__);                        \
        if (s.bs == 32) return FN<float, 32>(__VA_ARGS__);                        \
        return FN<float, 64>(__VA_ARGS__);                                        \
    } while (0)

hipError_t launch_attn_fwd(const AttnShape& s, const void* Q, const void* K, const void* V, void* O,
                           float* LSE, const int* row_ptr, const int* col_idx, hipStream_t st) {
    SPION_DISPATCH(fwd_t, s, Q, K, V, O, LSE, row_ptr, col_idx, st);
}

hipError_t launch_attn_bwd(const AttnShape& s, const void* Q, const void* K, const void* V,
                           const void* O, const void* dO, const float* LSE, void* dQ, void* dK,
                           void* dV, const int* row_ptr, const int* col_idx, const int* col_ptr,
                           const int* row_idx, int nnzb, void* workspace, hipStream_t st) {
    SPION_DISPATCH(bwd_t, s, Q, K, V, O, dO, LSE, dQ, dK, dV, row_ptr, col_idx, col_ptr, row_idx, nnzb,
                   workspace, st);
}

}  // namespace spion
