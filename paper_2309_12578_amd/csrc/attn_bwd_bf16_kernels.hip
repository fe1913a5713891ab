// bf16 block-sparse attention backward (the gradient of Eq. 5) tuned for gfx950, block size 32 or 64.
//
// One launch computes dQ, dK and dV.  Its grid holds two kinds of workgroups:
//   - query side: one workgroup per (head, block row I) walks the kept blocks of the row (BSR),
//     delta = rowsum(dO .* O), S^T and dP^T per block, dQ_I accumulated in registers;
//   - key side: one workgroup per (head, work item), a work item being a chunk of the kept rows of
//     one block column (BSC); S and dP per block, dK_J and dV_J accumulated in registers.
// The two sides share no data: the key side computes delta for the query rows of every block it
// visits from the O and dO tiles it loads (an MFMA whose diagonal is the row-wise dot product), so
// neither waits for the other, and workgroups of both kinds fill the machine together.  Block
// columns with more kept rows than one work item takes are cut into chunks that write fp32 partial
// tiles; a second, small launch adds them up in chunk order.  No atomics: gradients are bit-reproducible.
//
// Every workgroup finds its own work from the index: there is no work list to build, so nothing in
// the grid depends on another workgroup.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "attn_bf16_tiles.h"
#include "attn_common.h"
#include "spion_internal.h"

namespace spion {

// ------------------------------------------------------------------------------------------------
// Key-side work items, derived from col_ptr alone (the same list for every head).  A column with cnt
// kept rows is cut into nch = ceil(cnt / kChunk) near-equal chunks if cnt > kChunk, else it is one
// item (also when cnt == 0: its dK / dV must still be written as zeros).  Items are numbered with
// the chunks of split columns first, in column order (they are the longest and start first), then
// the unsplit columns in column order.  Chunk number w of that first group writes partial slot w.
// ------------------------------------------------------------------------------------------------
struct KeyItem {
    int J;      // block column, -1: no such item
    int kb, ke; // BSC entries [kb, ke)
    int slot;   // partial slot, -1: the item covers its whole column and writes dK / dV itself
};

__device__ __forceinline__ int lanes_below(unsigned long long mask) {
    return __builtin_amdgcn_mbcnt_hi((unsigned)(mask >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)mask, 0));
}

// All lanes of the calling wave must be active; the result is wave-uniform.
__device__ __forceinline__ KeyItem key_item_lookup(const int* __restrict__ col_ptr, int nb, int w, int lane) {
    KeyItem none = {-1, 0, 0, -1};
    int run = 0;   // chunks of split columns in the column groups before this one
    int c0_first = 0, cnt_first = 0;   // columns 0 .. 63, kept for the second search
    for (int base = 0; base < nb; base += 64) {
        const int J = base + lane;
        const bool valid = J < nb;
        const int c0 = valid ? col_ptr[J] : 0, cnt = valid ? col_ptr[J + 1] - c0 : 0;
        if (base == 0) {
            c0_first = c0;
            cnt_first = cnt;
        }
        const int nch = cnt > kChunk ? (cnt + kChunk - 1) / kChunk : 0;
        const int incl = wave_incl_scan(nch, lane);
        const int lo = run + incl - nch;
        const unsigned long long hit = __ballot(nch > 0 && w >= lo && w < lo + nch);
        if (hit) {
            const int src = __ffsll((long long)hit) - 1;
            const int c0s = __builtin_amdgcn_readlane(c0, src), cnts = __builtin_amdgcn_readlane(cnt, src);
            const int nchs = __builtin_amdgcn_readlane(nch, src);
            int ci = w - __builtin_amdgcn_readlane(lo, src);
            ci = ci < 0 ? 0 : (ci >= nchs ? nchs - 1 : ci);
            KeyItem it = {base + src, c0s + (ci * cnts) / nchs, c0s + ((ci + 1) * cnts) / nchs, w};
            return it;
        }
        run += __builtin_amdgcn_readlane(incl, 63);
    }
    int u = w - run;   // index among the unsplit columns
    for (int base = 0; base < nb; base += 64) {
        const int J = base + lane;
        const bool valid = J < nb;
        int c0 = c0_first, c1 = c0_first + cnt_first;
        if (base != 0) {
            c0 = valid ? col_ptr[J] : 0;
            c1 = valid ? col_ptr[J + 1] : 0;
        }
        const unsigned long long whole = __ballot(valid && c1 - c0 <= kChunk);
        const unsigned long long hit = __ballot(valid && c1 - c0 <= kChunk && lanes_below(whole) == u);
        if (hit) {
            const int src = __ffsll((long long)hit) - 1;
            KeyItem it = {base + src, __builtin_amdgcn_readlane(c0, src), __builtin_amdgcn_readlane(c1, src), -1};
            return it;
        }
        u -= __popcll(whole);
    }
    return none;
}

// The m-th split column: {J, first partial slot, chunks}; J < 0 if there are fewer.
__device__ __forceinline__ int4 split_column_lookup(const int* __restrict__ col_ptr, int nb, int m, int lane) {
    int run = 0;
    for (int base = 0; base < nb; base += 64) {
        const int J = base + lane;
        const bool valid = J < nb;
        const int cnt = valid ? col_ptr[J + 1] - col_ptr[J] : 0;
        const int nch = cnt > kChunk ? (cnt + kChunk - 1) / kChunk : 0;
        const int incl = wave_incl_scan(nch, lane);
        const unsigned long long split = __ballot(nch > 0);
        const unsigned long long hit = __ballot(nch > 0 && lanes_below(split) == m);
        if (hit) {
            const int src = __ffsll((long long)hit) - 1;
            const int nchs = __builtin_amdgcn_readlane(nch, src);
            return make_int4(base + src, run + __builtin_amdgcn_readlane(incl, src) - nchs, nchs, 0);
        }
        m -= __popcll(split);
        run += __builtin_amdgcn_readlane(incl, 63);
    }
    return make_int4(-1, 0, 0, 0);
}

// Own loads landed (up to `younger` younger ones may stay in flight: 0 or 4), previous LDS reads done,
// then meet the other waves.  A bare barrier: the fences of __syncthreads would wait for every load
// in flight, the prefetched blocks included.
__device__ __forceinline__ void tiles_ready(bool four_younger_in_flight) {
    if (four_younger_in_flight) __builtin_amdgcn_s_waitcnt(kWaitVm4);
    else __builtin_amdgcn_s_waitcnt(kWaitVm0);
    __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// ------------------------------------------------------------------------------------------------
// Grid layout.  Per head: key items [0, w_first), then the nb block rows, then key items
// [w_first, w_max); the long chunks of split columns come first so that they start first, the rows and
// the short columns fill in behind them.  With B H a multiple of 8 each XCD (own L2; workgroups
// are dealt to the XCDs round-robin) works on whole heads, items of all its heads interleaved.
// n_key_a / n_rows / n_key_c are the per-head counts of the three groups present in this launch
// (a group is absent when only one side is requested).
// ------------------------------------------------------------------------------------------------
template <int BS>
__global__ __launch_bounds__(BS * 4) void attn_bwd_bf16_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const bf16_t* __restrict__ O, const bf16_t* __restrict__ dO, const float* __restrict__ LSE,
    bf16_t* __restrict__ dQ, bf16_t* __restrict__ dK, bf16_t* __restrict__ dV,
    const int* __restrict__ row_ptr, const int* __restrict__ col_idx, const int* __restrict__ col_ptr,
    const int* __restrict__ row_idx, float* __restrict__ partial, int n_slots, int BH, int L, int nb,
    int n_key_a, int n_rows, int n_key_c, int w_first, float scale, float scale_log2) {
    constexpr int NT = BS / 16;   // 16-row tiles per block = waves per workgroup
    // Separate objects, so that the compiler can tell a read of one tile from a load in flight into
    // another and does not wait for it.  Query side: {ta, tb} hold {K, V} of a block, three stages
    // (0, 1, and {tc0, tc1}).  Key side: {ta, tb, tc} hold {Q, dO, O} of a block row, two stages.
    __shared__ __attribute__((aligned(16))) bf16_t ta0[BS * kD], tb0[BS * kD], tc0[BS * kD];
    __shared__ __attribute__((aligned(16))) bf16_t ta1[BS * kD], tb1[BS * kD], tc1[BS * kD];
    __shared__ __attribute__((aligned(16))) float lse0[BS], del0[BS], lse1[BS], del1[BS];

    const int tid = threadIdx.x, lane = tid & 63, r = lane & 15, g = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const SwzLane sl(r, g);
    const TileLoadLane tl(wave, lane);

    // which workgroup am I
    int x = 0, hpx = BH, l = blockIdx.x;
    if ((BH & 7) == 0) {
        x = blockIdx.x & 7;
        hpx = BH >> 3;
        l = blockIdx.x >> 3;
    }
    bool key_side;
    int bh, idx;   // idx: work item (key side) or block row (query side)
    if (l < hpx * n_key_a) {
        key_side = true;
        bh = x * hpx + l % hpx;
        idx = l / hpx;
    } else if (l < hpx * (n_key_a + n_rows)) {
        l -= hpx * n_key_a;
        key_side = false;
        bh = x * hpx + l / nb;
        idx = l % nb;
    } else {
        l -= hpx * (n_key_a + n_rows);
        key_side = true;
        bh = x * hpx + l % hpx;
        idx = w_first + l / hpx;
    }
    const size_t head = (size_t)bh * L * kD;
    const size_t vec = (size_t)bh * L;

    if (!key_side) {
        // ========================================================================================
        // query side: block row I, K / V tiles three stages deep (block it + 2 loads while block it
        // is multiplied)
        // ========================================================================================
        const int I = idx;
        const int qrow = I * BS + wave * 16 + r;
        auto issue = [&](bf16_t* kt, bf16_t* vt, int J) {
            tile_load_async(K + head + (size_t)J * BS * kD, kt, wave, tl);
            tile_load_async(V + head + (size_t)J * BS * kD, vt, wave, tl);
        };
        issue(ta0, tb0, I);   // the diagonal block, before any index is known
        bf16x8 qf[2], dof[2], of[2];
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const size_t off = head + (size_t)qrow * kD + c * 32 + g * 8;
            qf[c] = *reinterpret_cast<const bf16x8*>(Q + off);
            dof[c] = *reinterpret_cast<const bf16x8*>(dO + off);
            of[c] = *reinterpret_cast<const bf16x8*>(O + off);
        }
        const float lse2 = LSE[vec + qrow] * kLog2e;
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
            issue(ta0, tb0, first[0]);
        }
        // the second block goes out as soon as its index is known (a one-block row loads its block
        // twice: keeps the wait of step 0 uniform); it is the youngest load at step 0
        if (n > 0) issue(ta1, tb1, col_at(1));
        int Jnext = n > 0 ? col_at(2) : 0;   // block of step it + 2

        float delta = 0.f;
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int e = 0; e < 8; ++e) delta = fmaf((float)dof[c][e], (float)of[c][e], delta);
        delta = group_sum(delta);

        f32x4 dq[4];
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) dq[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

        auto step = [&](const bf16_t* kt, const bf16_t* vt, bf16_t* tk, bf16_t* tv, int it) {
            // in flight here: block `it` and block it + 1 (the four youngest loads; at step 0 whatever the
            // prologue loaded before them is waited for as well)
            tiles_ready(it + 1 < n || it == 0);
            if (it + 2 < n) issue(tk, tv, Jnext);
            Jnext = col_at(it + 3);
            // all K and V fragments are requested up front; the transposed K operands of the dQ product do
            // not depend on dS and are requested before the exponentials, so that they land under them
            bf16x8 kfr[NT][2], vfr[NT][2];
#pragma unroll
            for (int kt16 = 0; kt16 < NT; ++kt16)
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    kfr[kt16][c] = *reinterpret_cast<const bf16x8*>(kt + kt16 * 16 * kD + sl.frag[c]);
                    vfr[kt16][c] = *reinterpret_cast<const bf16x8*>(vt + kt16 * 16 * kD + sl.frag[c]);
                }
            f32x4 s[NT], dp[NT];
#pragma unroll
            for (int kt16 = 0; kt16 < NT; ++kt16) {
                // dP - delta comes out of the MFMA: the accumulator starts at -delta instead of 0
                s[kt16] = f32x4{0.f, 0.f, 0.f, 0.f};
                dp[kt16] = f32x4{-delta, -delta, -delta, -delta};
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    s[kt16] = mma_d(s[kt16], kfr[kt16][c], qf[c]);      // S^T = K Q^T
                    dp[kt16] = mma_d(dp[kt16], vfr[kt16][c], dof[c]);   // dP^T = V dO^T
                }
            }
            constexpr int NM = (BS / 32) * 4;
            bf16x8 kop[NM];
#pragma unroll
            for (int j = 0; j < NM; ++j) {
                const int o = sl.tr(j & 3) + (j >> 2) * 32 * kD;
                kop[j] = join(lds_read_tr(kt + o), lds_read_tr(kt + 16 * kD + o));
            }
            __builtin_amdgcn_sched_barrier(0);
            bf16x4 dsq[NT];
#pragma unroll
            for (int kt16 = 0; kt16 < NT; ++kt16) {
                f32x4 ds;
#pragma unroll
                for (int i = 0; i < 4; ++i) ds[i] = fast_exp2(fmaf(s[kt16][i], scale_log2, -lse2)) * dp[kt16][i];
                dsq[kt16] = to_quad<bf16_t>(ds);
            }
#pragma unroll
            for (int j = 0; j < NM; ++j) {
                const int pc = j >> 2;
                dq[j & 3] = mma_d(dq[j & 3], kop[j], join(dsq[2 * pc], dsq[2 * pc + 1]));   // dQ^T[d][query] += K^T dS^T
            }
        };

        for (int it = 0; it < n; it += 3) {
            step(ta0, tb0, tc0, tc1, it);
            if (it + 1 < n) step(ta1, tb1, ta0, tb0, it + 1);
            if (it + 2 < n) step(tc0, tc1, ta1, tb1, it + 2);
        }
        // an empty row never waited for its early load: it must land before this workgroup's LDS is freed
        __builtin_amdgcn_s_waitcnt(kWaitVm0);
        // Through a tile nobody reads any more: every wave is past the barrier of the last step, so only
        // the last block's stage can still be read; the wave's own 2 KB of any other tile were only ever
        // written by the wave's own loads, which have all landed.
        bf16_t* patch = (n % 3 == 1 ? ta1 : ta0) + wave * (16 * kD);   // last stage: (n - 1) % 3
        store_rows_coalesced(patch, dQ + head + (size_t)(I * BS + wave * 16) * kD, dq, scale, lane);
        return;
    }

    // ============================================================================================
    // key side: work item idx of head bh.  {Q, dO, O} tiles and LSE of a block row in two stages.
    // ============================================================================================
    const KeyItem item = key_item_lookup(col_ptr, nb, idx, lane);
    if (item.J < 0) return;
    const int J = item.J, n = item.ke - item.kb, slot = item.slot;
    const int krow = J * BS + wave * 16 + r;
    const int last = n > 0 ? n - 1 : 0;
    // the item's block rows, one per lane (an item has at most kChunk <= 64 of them): read once, so that
    // no scalar load is in flight inside the steps (scalar loads return out of order, and while one is
    // outstanding every wait for an LDS read has to wait for all of them)
    static_assert(kChunk <= 64, "a key-side work item must fit one wave's lanes");
    const int rows_v = n > 0 ? row_idx[item.kb + (lane < last ? lane : last)] : 0;
    auto row_at = [&](int t) { return __builtin_amdgcn_readlane(rows_v, t < last ? t : last); };

    // six tile loads per wave, plus one 4-byte-per-lane load of LSE in wave 0
    auto issue = [&](bf16_t* qt, bf16_t* dt_, bf16_t* ot, float* lse_s, int I) {
        tile_load_async(Q + head + (size_t)I * BS * kD, qt, wave, tl);
        tile_load_async(dO + head + (size_t)I * BS * kD, dt_, wave, tl);
        tile_load_async(O + head + (size_t)I * BS * kD, ot, wave, tl);
        if (wave == 0 && lane < BS)
            __builtin_amdgcn_global_load_lds(LSE + vec + (size_t)I * BS + lane, (lds_void_ptr)lse_s, 4, 0, 0);
    };
    int Inext = 0;   // block row of step it + 1
    if (n > 0) {
        issue(ta0, tb0, tc0, lse0, row_at(0));
        Inext = row_at(1);
    }
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

    auto step = [&](const bf16_t* qt, const bf16_t* dt_, const bf16_t* ot, float* lse_s, float* del_s,
                    bf16_t* nq, bf16_t* nd, bf16_t* no, float* nlse, int it) {
        // everyone's part of block `it` has landed and the other stage is no longer read
        tiles_ready(false);
        if (it + 1 < n) issue(nq, nd, no, nlse, Inext);
        Inext = row_at(it + 2);
        // delta of the 16 query rows 16 wave .. + 15: the diagonal of dO O^T; stored negated, it seeds
        // the dP accumulators below.  Wave 0 also turns LSE into log2 units.
        {
            f32x4 dd = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const int off = wave * 16 * kD + sl.frag[c];
                dd = mma_d(dd, *reinterpret_cast<const bf16x8*>(dt_ + off), *reinterpret_cast<const bf16x8*>(ot + off));
            }
            // lane (r, g) holds (dO O^T)[4 g + i][r]: the diagonal entry of row r sits in lane group r / 4
            const float a = (r & 1) ? dd[1] : dd[0], b = (r & 1) ? dd[3] : dd[2];
            if (g == (r >> 2)) del_s[wave * 16 + r] = -((r & 2) ? b : a);
            if (wave == 0 && lane < BS) lse_s[lane] *= kLog2e;
        }
        lds_barrier();
        // 32 query rows at a time: S and dP of two 16-row tiles, then their share of dV and dK, so that
        // only two tiles' worth of P and dS are live; LDS operands are requested one MFMA group ahead
        bf16x8 fq[2], fd[2];
        auto frags = [&](int qt16) {
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                fq[c] = *reinterpret_cast<const bf16x8*>(qt + qt16 * 16 * kD + sl.frag[c]);
                fd[c] = *reinterpret_cast<const bf16x8*>(dt_ + qt16 * 16 * kD + sl.frag[c]);
            }
        };
        auto opnd = [&](int pc, int j) {   // transposed operand of MFMA j of this 32-row group
            const bf16_t* tile = (j & 1) ? qt : dt_;
            const int o = sl.tr(j >> 1) + pc * 32 * kD;
            return join(lds_read_tr(tile + o), lds_read_tr(tile + 16 * kD + o));
        };
        frags(0);
#pragma unroll
        for (int pc = 0; pc < NT / 2; ++pc) {
            bf16x4 pq[2], dsq[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int qt16 = 2 * pc + h;
                f32x4 s = f32x4{0.f, 0.f, 0.f, 0.f};
                f32x4 dp = *reinterpret_cast<const f32x4*>(&del_s[qt16 * 16 + 4 * g]);   // -delta: the MFMA returns dP - delta
                const f32x4 lse4 = *reinterpret_cast<const f32x4*>(&lse_s[qt16 * 16 + 4 * g]);   // log2 units
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    s = mma_d(s, fq[c], kf[c]);     // S = Q K^T
                    dp = mma_d(dp, fd[c], vf[c]);   // dP = dO V^T
                }
                __builtin_amdgcn_sched_barrier(0);
                if (qt16 + 1 < NT) frags(qt16 + 1);   // lands while the exponentials below run
                __builtin_amdgcn_sched_barrier(0);
                f32x4 p, ds;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    p[i] = fast_exp2(fmaf(s[i], scale_log2, -lse4[i]));
                    ds[i] = p[i] * dp[i];
                }
                pq[h] = to_quad<bf16_t>(p);
                dsq[h] = to_quad<bf16_t>(ds);
            }
            // dV^T[d][key] += dO^T P and dK^T[d][key] += Q^T dS for these 32 rows, interleaved
            const bf16x8 pf = join(pq[0], pq[1]), dsf = join(dsq[0], dsq[1]);
            bf16x8 ring[2];
            ring[0] = opnd(pc, 0);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if (j + 1 < 8) ring[(j + 1) & 1] = opnd(pc, j + 1);
                __builtin_amdgcn_sched_barrier(0);
                if (j & 1) dk[j >> 1] = mma_d(dk[j >> 1], ring[j & 1], dsf);
                else dv[j >> 1] = mma_d(dv[j >> 1], ring[j & 1], pf);
            }
        }
    };

    for (int it = 0; it < n; it += 2) {
        step(ta0, tb0, tc0, lse0, del0, ta1, tb1, tc1, lse1, it);
        if (it + 1 < n) step(ta1, tb1, tc1, lse1, del1, ta0, tb0, tc0, lse0, it + 1);
    }
    __builtin_amdgcn_s_waitcnt(kWaitVm0);   // the owned fragments of a column without kept rows

    if (slot < 0) {
        // Through the stage the last block did not use: every wave is past the first barrier of the last
        // step, i.e. done reading that stage, no load targets it any more, and the only loads that ever
        // touched this wave's 2 KB of its tiles were the wave's own.
        const bool odd = (n & 1) != 0;   // last block in stage 0 -> stage 1 is free
        bf16_t* pa = (odd ? ta1 : ta0) + wave * (16 * kD);
        bf16_t* pb = (odd ? tb1 : tb0) + wave * (16 * kD);
        const size_t row0 = head + (size_t)(J * BS + wave * 16) * kD;
        store_rows_coalesced(pa, dK + row0, dk, scale, lane);
        store_rows_coalesced(pb, dV + row0, dv, 1.f, lane);
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
}

// Adds the partial tiles of every split block column, in chunk order.  Workgroup = (head, m-th split
// column, part): 256 threads, one float4 of the output tile each, bs / 16 parts per tile, so that the
// loads of all chunks of a float4 are in flight together.
template <int BS>
__global__ __launch_bounds__(256) void attn_bwd_bf16_reduce_kernel(
    const float* __restrict__ partial, const int* __restrict__ col_ptr, int nb, int split_max, int n_slots,
    bf16_t* __restrict__ dK, bf16_t* __restrict__ dV, int L, float scale) {
    constexpr int PARTS = BS / 16;
    const int part = blockIdx.x % PARTS, m = (blockIdx.x / PARTS) % split_max;
    const int bh = blockIdx.x / (PARTS * split_max);
    const int4 info = split_column_lookup(col_ptr, nb, m, threadIdx.x & 63);   // {J, first slot, chunks}
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
    store_quad<bf16_t>(dK + out, ak * scale);
    store_quad<bf16_t>(dV + out, av);
}

// ------------------------------------------------------------------------------------------------
// launcher (called by the dispatch in attn_kernels.hip).  phases: bit 0 query side, bit 1 key side.
// ------------------------------------------------------------------------------------------------
template <int BS>
hipError_t bwd_bf16(const AttnShape& s, const void* Q, const void* K, const void* V, const void* O,
                    const void* dO, const float* LSE, void* dQ, void* dK, void* dV, const int* row_ptr,
                    const int* col_idx, const int* col_ptr, const int* row_idx, int nnzb, int w_max,
                    int split_max, int n_slots, float* partial, hipStream_t st) {
    const bool rows = (s.bwd_phases & 1) != 0, keys = (s.bwd_phases & 2) != 0;
    // the chunks of split columns are the first work items; about nnzb / kChunk of them
    int w_first = nnzb / kChunk + 1;
    if (w_first > w_max) w_first = w_max;
    const int n_key_a = keys ? w_first : 0, n_rows = rows ? s.nb : 0, n_key_c = keys ? w_max - w_first : 0;
    const long long total = (long long)s.BH * (n_key_a + n_rows + n_key_c);
    if (total > 0) {
        attn_bwd_bf16_kernel<BS><<<dim3((unsigned)total), dim3(BS * 4), 0, st>>>(
            static_cast<const bf16_t*>(Q), static_cast<const bf16_t*>(K), static_cast<const bf16_t*>(V),
            static_cast<const bf16_t*>(O), static_cast<const bf16_t*>(dO), LSE, static_cast<bf16_t*>(dQ),
            static_cast<bf16_t*>(dK), static_cast<bf16_t*>(dV), row_ptr, col_idx, col_ptr, row_idx, partial,
            n_slots, s.BH, s.L, s.nb, n_key_a, n_rows, n_key_c, w_first, s.scale, s.scale * kLog2e);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (keys && split_max > 0) {
        attn_bwd_bf16_reduce_kernel<BS><<<dim3((unsigned)(split_max * s.BH * (BS / 16))), dim3(256), 0, st>>>(
            partial, col_ptr, s.nb, split_max, n_slots, static_cast<bf16_t*>(dK), static_cast<bf16_t*>(dV), s.L,
            s.scale);
    }
    return hipGetLastError();
}

template hipError_t bwd_bf16<32>(const AttnShape&, const void*, const void*, const void*, const void*,
                                 const void*, const float*, void*, void*, void*, const int*, const int*,
                                 const int*, const int*, int, int, int, int, float*, hipStream_t);
template hipError_t bwd_bf16<64>(const AttnShape&, const void*, const void*, const void*, const void*,
                                 const void*, const float*, void*, void*, void*, const int*, const int*,
                                 const int*, const int*, int, int, int, int, float*, hipStream_t);

}  // namespace spion
