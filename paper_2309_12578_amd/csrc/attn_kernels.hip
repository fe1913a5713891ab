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

#include "spion_internal.h"

namespace spion {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kD = 64;  // head dimension
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Per element type: a 16-byte lane fragment of EPL elements; four lane groups make a chunk of KC
// contraction elements along d.
template <typename T>
struct Elem;
template <>
struct Elem<float> {
    static constexpr int EPL = 4, KC = 16;
    typedef f32x4 Frag;   // d-chunk fragment
    typedef f32x4 Quad;   // 4 consecutive elements (one accumulator tile's worth per lane)
};
template <>
struct Elem<bf16_t> {
    static constexpr int EPL = 8, KC = 32;
    typedef bf16x8 Frag;
    typedef bf16x4 Quad;
};

// acc[16x16] += A(16 x KC) * B(KC x 16), both fragments indexed [lane % 16][chunk + (lane / 16) * EPL + e]
__device__ __forceinline__ f32x4 mma_d(f32x4 acc, bf16x8 a, bf16x8 b) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc, 0, 0, 0);
}
__device__ __forceinline__ f32x4 mma_d(f32x4 acc, f32x4 a, f32x4 b) {
#pragma unroll
    for (int i = 0; i < 4; ++i) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[i], b[i], acc, 0, 0, 0);
    return acc;
}
// 16-deep contraction: lane group g holds contraction indices 4 g .. 4 g + 3
__device__ __forceinline__ f32x4 mma_q(f32x4 acc, bf16x4 a, bf16x4 b) {
    return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, a),
                                                     __builtin_bit_cast(s16x4, b), acc, 0, 0, 0);
}
__device__ __forceinline__ f32x4 mma_q(f32x4 acc, f32x4 a, f32x4 b) { return mma_d(acc, a, b); }

template <typename T>
__device__ __forceinline__ typename Elem<T>::Quad to_quad(f32x4 v);
template <>
__device__ __forceinline__ f32x4 to_quad<float>(f32x4 v) {
    return v;
}
template <>
__device__ __forceinline__ bf16x4 to_quad<bf16_t>(f32x4 v) {
    bf16x4 r;
    r[0] = (bf16_t)v[0];
    r[1] = (bf16_t)v[1];
    r[2] = (bf16_t)v[2];
    r[3] = (bf16_t)v[3];
    return r;
}
__device__ __forceinline__ bf16x8 join(bf16x4 lo, bf16x4 hi) {
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// acc[dt] += T^T(16 d-rows x keys) * X(keys x 16 owned rows) for dt = 0..3, where
//   tl      transposed tile in LDS, [64][LDT], element (d, key)
//   x[kt]   accumulator-layout tiles (16 keys each) already converted to the element type
// i.e. out^T[d][owned] += sum_key tile[key][d] * x[key][owned].
template <typename T, int BS, int LDT>
__device__ __forceinline__ void mma_over_rows(f32x4 (&acc)[4], const T* tl,
                                              const typename Elem<T>::Quad (&x)[BS / 16], int r, int g) {
    typedef typename Elem<T>::Quad Quad;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
        const T* row = tl + (dt * 16 + r) * LDT + 4 * g;
        if constexpr (sizeof(T) == 2 && BS >= 32) {
#pragma unroll
            for (int pc = 0; pc < BS / 32; ++pc) {
                const bf16x4 lo = *reinterpret_cast<const bf16x4*>(row + pc * 32);
                const bf16x4 hi = *reinterpret_cast<const bf16x4*>(row + pc * 32 + 16);
                acc[dt] = mma_d(acc[dt], join(lo, hi), join(x[2 * pc], x[2 * pc + 1]));
            }
        } else {
#pragma unroll
            for (int kt = 0; kt < BS / 16; ++kt) {
                const Quad a = *reinterpret_cast<const Quad*>(row + kt * 16);
                acc[dt] = mma_q(acc[dt], a, x[kt]);
            }
        }
    }
}

// Stage one bs x 64 tile (contiguous in global memory) into LDS: row-major into rm (if non-null
// at compile time) and transposed into tr.
template <typename T, int BS, int LDK, int LDT, bool ROWMAJOR, bool TRANSPOSED>
__device__ __forceinline__ void stage_tile(const T* __restrict__ src, T* rm, T* tr, int tid) {
    typedef typename Elem<T>::Frag Frag;
    constexpr int EPL = Elem<T>::EPL;
    constexpr int NT = BS * 4;
    constexpr int FPR = kD / EPL;  // fragments per row
#pragma unroll
    for (int it = 0; it < (int)sizeof(T); ++it) {
        const int idx = it * NT + tid;
        const int row = idx / FPR, cc = idx % FPR;
        const Frag f = *reinterpret_cast<const Frag*>(src + (size_t)idx * EPL);
        if constexpr (ROWMAJOR) *reinterpret_cast<Frag*>(rm + row * LDK + cc * EPL) = f;
        if constexpr (TRANSPOSED) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) tr[(cc * EPL + e) * LDT + row] = f[e];
        }
    }
}

__device__ __forceinline__ float group_max(float v) {
    v = fmaxf(v, __shfl_xor(v, 16));
    return fmaxf(v, __shfl_xor(v, 32));
}
__device__ __forceinline__ float group_sum(float v) {
    v += __shfl_xor(v, 16);
    return v + __shfl_xor(v, 32);
}

template <typename T>
__device__ __forceinline__ void store_quad(T* dst, f32x4 v) {
    *reinterpret_cast<typename Elem<T>::Quad*>(dst) = to_quad<T>(v);
}

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
    if (paper_denom) {
        // Algorithm 6: every masked entry of the row counts as a score of 0
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
// Key-side work list.  Vertical stripes give block columns with up to nb kept rows next to columns
// with one or two, so the key-side kernel does not take one column per workgroup: a column with cnt
// kept rows is cut into nch = ceil(cnt / kChunk) near-equal chunks, each a work item.  A column with
// one chunk writes dK / dV directly; the chunks of a longer column write fp32 partial tiles into
// numbered slots that a second kernel adds up in chunk order (deterministic).  The list is the same
// for every head; one wave of the query-side kernel (which always runs first) builds it.
//   sched[w]   = {J, kb, ke, slot}: BSC entries [kb, ke) of column J; slot < 0: write final output;
//                J < 0: unused work item
//   colinfo[J] = {first slot, nch}
// ------------------------------------------------------------------------------------------------
constexpr int kChunk = 8;

__host__ __device__ inline int key_work_items_max(int nnzb, int nb) { return nnzb / kChunk + nb; }
__host__ __device__ inline int key_slots_max(int nnzb) { return 2 * (nnzb / kChunk) + 2; }

__device__ __forceinline__ int wave_incl_scan(int v, int lane) {
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_up(v, off);
        if (lane >= off) v += o;
    }
    return v;
}

__device__ void build_key_schedule(const int* __restrict__ col_ptr, int nb, int w_max,
                                   int4* __restrict__ sched, int2* __restrict__ colinfo, int lane) {
    int run_w = 0, run_s = 0;
    for (int base = 0; base < nb; base += 64) {
        const int J = base + lane;
        const bool valid = J < nb;
        const int c0 = valid ? col_ptr[J] : 0;
        const int cnt = valid ? col_ptr[J + 1] - c0 : 0;
        const int nch = valid ? (cnt > kChunk ? (cnt + kChunk - 1) / kChunk : 1) : 0;
        const int ns = nch > 1 ? nch : 0;
        const int w_incl = wave_incl_scan(nch, lane), s_incl = wave_incl_scan(ns, lane);
        const int w0 = run_w + w_incl - nch, s0 = run_s + s_incl - ns;
        if (valid) {
            colinfo[J] = make_int2(nch > 1 ? s0 : -1, nch);
            for (int ci = 0; ci < nch && w0 + ci < w_max; ++ci)
                sched[w0 + ci] = make_int4(J, c0 + (ci * cnt) / nch, c0 + ((ci + 1) * cnt) / nch,
                                           nch > 1 ? s0 + ci : -1);
        }
        run_w += __shfl(w_incl, 63);
        run_s += __shfl(s_incl, 63);
    }
    for (int w = run_w + lane; w < w_max; w += 64) sched[w] = make_int4(-1, 0, 0, -1);
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
    const int* __restrict__ col_ptr, int w_max, int4* __restrict__ sched, int2* __restrict__ colinfo,
    int L, int nb, float scale, float scale_log2) {
    if (blockIdx.x == 0 && threadIdx.x < 64)
        build_key_schedule(col_ptr, nb, w_max, sched, colinfo, threadIdx.x);
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
// workgroup = (head, block column J); thread t owns float4 number t, t + NT, ... of the tile.
template <typename T, int BS>
__global__ __launch_bounds__(BS * 4) void attn_bwd_dkv_reduce_kernel(
    const float* __restrict__ partial, const int2* __restrict__ colinfo, int n_slots, T* __restrict__ dK,
    T* __restrict__ dV, int L, int nb, float scale) {
    const int J = blockIdx.x % nb, bh = blockIdx.x / nb;
    const int2 info = colinfo[J];
    if (info.y <= 1) return;
    constexpr int NT = BS * 4, NV = BS * kD / 4;
    const float* base = partial + ((size_t)bh * n_slots + info.x) * (2 * BS * kD);
    const size_t out0 = (size_t)bh * L * kD + (size_t)J * BS * kD;
    for (int v = threadIdx.x; v < NV; v += NT) {
        f32x4 ak = f32x4{0.f, 0.f, 0.f, 0.f}, av = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int c = 0; c < info.y; ++c) {
            const float* pk = base + (size_t)c * (2 * BS * kD);
            ak += *reinterpret_cast<const f32x4*>(pk + v * 4);
            av += *reinterpret_cast<const f32x4*>(pk + BS * kD + v * 4);
        }
        store_quad<T>(dK + out0 + v * 4, ak * scale);
        store_quad<T>(dV + out0 + v * 4, av);
    }
}

// ------------------------------------------------------------------------------------------------
// host launchers
// ------------------------------------------------------------------------------------------------
size_t attn_bwd_workspace_bytes(int BH, int L, int bs, int nb, int nnzb) {
    const BwdWorkspace ws(BH, L, bs, nb, nnzb);
    return ws.total;
}

BwdWorkspace::BwdWorkspace(int BH, int L, int bs, int nb, int nnzb) {
    auto up = [](size_t x) { return (x + 255) / 256 * 256; };
    w_max = key_work_items_max(nnzb, nb);
    n_slots = key_slots_max(nnzb);
    delta_off = 0;
    sched_off = delta_off + up((size_t)BH * L * sizeof(float));
    colinfo_off = sched_off + up((size_t)w_max * sizeof(int4));
    partial_off = colinfo_off + up((size_t)nb * sizeof(int2));
    total = partial_off + up((size_t)BH * n_slots * 2 * bs * kD * sizeof(float));
}

template <typename T, int BS>
static hipError_t fwd_t(const AttnShape& s, const void* Q, const void* K, const void* V, void* O,
                        float* LSE, const int* row_ptr, const int* col_idx, hipStream_t st) {
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
    int2* colinfo = reinterpret_cast<int2*>(base + ws.colinfo_off);
    float* partial = reinterpret_cast<float*>(base + ws.partial_off);
    const dim3 block(BS * 4);
    if (s.bwd_phases & 1) {
        attn_bwd_dq_kernel<T, BS><<<dim3((unsigned)(s.nb * s.BH)), block, 0, st>>>(
            static_cast<const T*>(Q), static_cast<const T*>(K), static_cast<const T*>(V),
            static_cast<const T*>(O), static_cast<const T*>(dO), LSE, static_cast<T*>(dQ), delta,
            row_ptr, col_idx, col_ptr, ws.w_max, sched, colinfo, s.L, s.nb, s.scale, s.scale * kLog2e);
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
        attn_bwd_dkv_reduce_kernel<T, BS><<<dim3((unsigned)(s.nb * s.BH)), block, 0, st>>>(
            partial, colinfo, ws.n_slots, static_cast<T*>(dK), static_cast<T*>(dV), s.L, s.nb, s.scale);
    }
    return hipGetLastError();
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
