// Device helpers shared by the attention kernels: MFMA wrappers, fragment types, wave-level
// reductions and the key-side work list of the backward pass.
#ifndef SPION_ATTN_COMMON_H_
#define SPION_ATTN_COMMON_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

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

// Reductions over the four lanes r, r + 16, r + 32, r + 48 that hold values of the same owned row.
// v_permlane16_swap / v_permlane32_swap exchange rows of 16 (halves of 32) lanes between two
// registers in the VALU: with both registers holding v, one comes back as {row 0, row 0, row 2,
// row 2} and the other as {row 1, row 1, row 3, row 3} (resp. low half twice / high half twice).
// No LDS round trip, unlike a shuffle.  The two results pass through an empty asm statement: given
// equal inputs the compiler otherwise treats them as equal and drops the combine.
__device__ __forceinline__ void swap_rows16(float v, float& a, float& b) {
    const unsigned u = __builtin_bit_cast(unsigned, v);
    const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    unsigned r0 = r[0], r1 = r[1];
    asm volatile("" : "+v"(r0), "+v"(r1));
    a = __builtin_bit_cast(float, r0);
    b = __builtin_bit_cast(float, r1);
}
__device__ __forceinline__ void swap_halves32(float v, float& a, float& b) {
    const unsigned u = __builtin_bit_cast(unsigned, v);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    unsigned r0 = r[0], r1 = r[1];
    asm volatile("" : "+v"(r0), "+v"(r1));
    a = __builtin_bit_cast(float, r0);
    b = __builtin_bit_cast(float, r1);
}
__device__ __forceinline__ float group_max(float v) {
    float a, b;
    swap_rows16(v, a, b);
    swap_halves32(fmaxf(a, b), a, b);
    return fmaxf(a, b);
}
__device__ __forceinline__ float group_sum(float v) {
    float a, b;
    swap_rows16(v, a, b);
    swap_halves32(a + b, a, b);
    return a + b;
}

template <typename T>
__device__ __forceinline__ void store_quad(T* dst, f32x4 v) {
    *reinterpret_cast<typename Elem<T>::Quad*>(dst) = to_quad<T>(v);
}

// ------------------------------------------------------------------------------------------------
// Key-side work items.  Vertical stripes give block columns with up to nb kept rows next to columns
// with one or two, so the key side does not take one column per workgroup: a column with cnt kept
// rows is cut into nch = ceil(cnt / kChunk) near-equal chunks, each a work item.  A column with one
// chunk writes dK / dV directly; the chunks of a longer column write fp32 partial tiles into numbered
// slots that a second kernel adds up in chunk order (deterministic).  The list is the same for every
// head.  The generic kernels read it from the workspace, where one wave of their query-side kernel
// (which runs first) builds it:
//   sched[w]   = {J, kb, ke, slot}: BSC entries [kb, ke) of column J; slot < 0: write final output;
//                J < 0: unused work item
//   sched[w_max + w] = the first four block rows of the item (unused by the generic kernels)
//   split[m]   = {J, first slot, nch, 0} for the m-th split column; J < 0: unused entry
// The tuned bf16 backward derives the same items in every workgroup from col_ptr instead.
// ------------------------------------------------------------------------------------------------
#ifndef SPION_KEY_CHUNK
#define SPION_KEY_CHUNK 16   // kept rows per key-side work item (build-time tunable; 10-16 measure alike,
                             // shorter chunks cost partial-tile traffic, longer ones the longest chain)
#endif
constexpr int kChunk = SPION_KEY_CHUNK;

__host__ __device__ inline int key_work_items_max(int nnzb, int nb) { return nnzb / kChunk + nb; }
__host__ __device__ inline int key_slots_max(int nnzb) { return 2 * (nnzb / kChunk) + 2; }
__host__ __device__ inline int key_split_max(int nnzb) { return nnzb / (kChunk + 1) + 1; }

// Inclusive prefix sum over the wave with DPP moves (VALU speed, no LDS crossbar): shifts of 1, 2, 4, 8
// inside each row of 16 lanes, then lane 15 of rows 0 and 2 added to rows 1 and 3, then lane 31 added
// to rows 2 and 3.  A lane whose source is outside its row, or whose row is masked off, adds the 0
// given as old value.  All lanes must be active.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_fetch0(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, ROW_MASK, 0xf, false);
}
__device__ __forceinline__ int wave_incl_scan(int v, int /*lane*/) {
    v += dpp_fetch0<0x111, 0xf>(v);   // row_shr:1
    v += dpp_fetch0<0x112, 0xf>(v);   // row_shr:2
    v += dpp_fetch0<0x114, 0xf>(v);   // row_shr:4
    v += dpp_fetch0<0x118, 0xf>(v);   // row_shr:8
    v += dpp_fetch0<0x142, 0xa>(v);   // row_bcast:15 into rows 1 and 3
    v += dpp_fetch0<0x143, 0xc>(v);   // row_bcast:31 into rows 2 and 3
    return v;
}

__device__ void build_key_schedule(const int* __restrict__ col_ptr, const int* __restrict__ row_idx, int nb,
                                   int w_max, int split_max, int4* __restrict__ sched,
                                   int4* __restrict__ split, int lane) {
    // Two passes: the chunks of split columns (the longest work items) get the lowest work item
    // numbers and so start first; columns that fit one work item follow.
    int run_w = 0, run_s = 0, run_m = 0;
    for (int pass = 0; pass < 2; ++pass) {
        for (int base = 0; base < nb; base += 64) {
            const int J = base + lane;
            const bool valid = J < nb;
            const int c0 = valid ? col_ptr[J] : 0;
            const int cnt = valid ? col_ptr[J + 1] - c0 : 0;
            const int nch_all = valid ? (cnt > kChunk ? (cnt + kChunk - 1) / kChunk : 1) : 0;
            const bool mine = valid && ((nch_all > 1) == (pass == 0));
            const int nch = mine ? nch_all : 0;
            const int ns = nch > 1 ? nch : 0, is_split = nch > 1 ? 1 : 0;
            const int w_incl = wave_incl_scan(nch, lane), s_incl = wave_incl_scan(ns, lane);
            const int m_incl = wave_incl_scan(is_split, lane);
            const int w0 = run_w + w_incl - nch, s0 = run_s + s_incl - ns, m0 = run_m + m_incl - is_split;
            if (mine) {
                if (is_split && m0 < split_max) split[m0] = make_int4(J, s0, nch, 0);
                for (int ci = 0; ci < nch && w0 + ci < w_max; ++ci) {
                    const int kb = c0 + (ci * cnt) / nch, ke = c0 + ((ci + 1) * cnt) / nch;
                    sched[w0 + ci] = make_int4(J, kb, ke, nch > 1 ? s0 + ci : -1);
                    int fr[4] = {0, 0, 0, 0};
                    if (ke > kb) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) fr[e] = row_idx[kb + e < ke - 1 ? kb + e : ke - 1];
                    }
                    sched[w_max + w0 + ci] = make_int4(fr[0], fr[1], fr[2], fr[3]);
                }
            }
            run_w += __shfl(w_incl, 63);
            run_s += __shfl(s_incl, 63);
            run_m += __shfl(m_incl, 63);
        }
    }
    for (int w = run_w + lane; w < w_max; w += 64) sched[w] = make_int4(-1, 0, 0, -1);
    for (int m = run_m + lane; m < split_max; m += 64) split[m] = make_int4(-1, 0, 0, 0);
}

}  // namespace spion
#endif
