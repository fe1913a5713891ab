// Pattern generation kernels for gfx950 (Algorithm 3 and Algorithm 4 of the SPION paper).
//
//   conv_pool_kernel      Eq. 3 + Eq. 4 fused: one streaming pass over A^s that scatters every
//                         (fixed-point) score into the <= 7 pooled blocks its diagonal filter window
//                         touches.  HBM bound: A^s is read exactly once, nothing L x L is written.
//   pattern_finish_kernel one workgroup: threshold (exact order statistic / mean + k std),
//                         successor bits, anti-diagonal wavefront flood fill, forced diagonal,
//                         BSR + BSC compaction.  Latency bound (nb^2 <= ~1M cells).
//
// Arithmetic: a_q = rint(a * 2^40) in int64; all sums are integer, so any summation order (tiling,
// atomics) gives the same bits.  This file is compiled with -ffp-contract=off: the fp64 mean / std
// threshold must round exactly as its sequential definition.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "spion_internal.h"

namespace spion {

// ------------------------------------------------------------------------------------------------
// conv + pool
// ------------------------------------------------------------------------------------------------
// Input block (I, J) of A^s (bs x bs scores).  conv_out(i, j) = sum_{g=-p..p} a(i+g, j+g), so the
// score at local position (u, v) of this block is added to the outputs (u-g, v-g), g in [-p, p].
// Those outputs fall into blocks (I+di, J+dj) with di, dj in {-1, 0, +1} (p <= bs) and never into
// (-1,+1) or (+1,-1) because g shifts both coordinates alike.  The number of g landing in
// (di, dj) is the size of an interval intersection, a small integer weight; the block
// contributes sum(weight * a_q) to each of its 7 possible targets.
//
// g-intervals for a local coordinate x in [0, bs): block offset -1: [x+1, p], 0: [max(x-bs+1,-p),
// min(x,p)], +1: [-p, x-bs].
__device__ __forceinline__ int isect(int lo_a, int hi_a, int lo_b, int hi_b) {
    const int lo = lo_a > lo_b ? lo_a : lo_b;
    const int hi = hi_a < hi_b ? hi_a : hi_b;
    const int n = hi - lo + 1;
    return n > 0 ? n : 0;
}

__device__ __forceinline__ long long wave_sum_i64(long long v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

constexpr int kConvThreads = 256;

// grid.x = nb * nb input blocks; block = 256 threads; bs in {16, 32, 64} (bs % 4 == 0).
__global__ __launch_bounds__(kConvThreads) void conv_pool_kernel(const float* __restrict__ A, int L,
                                                                  int bs, int p,
                                                                  unsigned long long* __restrict__ pool) {
    const int nb = L / bs;
    const int I = blockIdx.x / nb, J = blockIdx.x % nb;
    const int tid = threadIdx.x;
    const int vec_per_row = bs >> 2;             // float4 per block row
    const int n_vec = bs * vec_per_row;          // float4 in the block

    long long acc[7] = {0, 0, 0, 0, 0, 0, 0};   // (0,0) (-1,-1) (+1,+1) (-1,0) (0,-1) (+1,0) (0,+1)
    const float* base = A + (size_t)I * bs * L + (size_t)J * bs;
    for (int idx = tid; idx < n_vec; idx += kConvThreads) {
        const int u = idx / vec_per_row;
        const int v0 = (idx % vec_per_row) << 2;
        const float4 a4 = *reinterpret_cast<const float4*>(base + (size_t)u * L + v0);
        const float av[4] = {a4.x, a4.y, a4.z, a4.w};
        // row intervals
        const int rm_lo = u + 1, rm_hi = p;                                   // di = -1
        const int r0_lo = (u - bs + 1) > -p ? (u - bs + 1) : -p, r0_hi = u < p ? u : p;  // di = 0
        const int rp_lo = -p, rp_hi = u - bs;                                 // di = +1
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int v = v0 + e;
            const long long aq = __double2ll_rn((double)av[e] * 1099511627776.0);
            const int cm_lo = v + 1, cm_hi = p;
            const int c0_lo = (v - bs + 1) > -p ? (v - bs + 1) : -p, c0_hi = v < p ? v : p;
            const int cp_lo = -p, cp_hi = v - bs;
            acc[0] += (long long)isect(r0_lo, r0_hi, c0_lo, c0_hi) * aq;
            acc[1] += (long long)isect(rm_lo, rm_hi, cm_lo, cm_hi) * aq;
            acc[2] += (long long)isect(rp_lo, rp_hi, cp_lo, cp_hi) * aq;
            acc[3] += (long long)isect(rm_lo, rm_hi, c0_lo, c0_hi) * aq;
            acc[4] += (long long)isect(r0_lo, r0_hi, cm_lo, cm_hi) * aq;
            acc[5] += (long long)isect(rp_lo, rp_hi, c0_lo, c0_hi) * aq;
            acc[6] += (long long)isect(r0_lo, r0_hi, cp_lo, cp_hi) * aq;
        }
    }

    __shared__ long long part[kConvThreads / 64][7];
    const int wave = tid >> 6, lane = tid & 63;
#pragma unroll
    for (int t = 0; t < 7; ++t) {
        const long long s = wave_sum_i64(acc[t]);
        if (lane == 0) part[wave][t] = s;
    }
    __syncthreads();
    if (tid < 7) {
        long long s = 0;
#pragma unroll
        for (int w = 0; w < kConvThreads / 64; ++w) s += part[w][tid];
        const int di_tab[7] = {0, -1, 1, -1, 0, 1, 0};
        const int dj_tab[7] = {0, -1, 1, 0, -1, 0, 1};
        const int ti = I + di_tab[tid], tj = J + dj_tab[tid];
        if (s != 0 && ti >= 0 && ti < nb && tj >= 0 && tj < nb)
            atomicAdd(&pool[(size_t)ti * nb + tj], (unsigned long long)s);
    }
}

__global__ void zero_u64_kernel(unsigned long long* __restrict__ p, size_t n) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0ull;
}

// ------------------------------------------------------------------------------------------------
// threshold + fill + compaction (one workgroup)
// ------------------------------------------------------------------------------------------------
constexpr int kFinishThreads = 1024;
constexpr unsigned kDown = 1u, kRight = 2u, kDiag = 4u;

struct Thresh {
    int is_int;
    long long ti;
    double td;
};

__device__ __forceinline__ bool above(long long x, const Thresh& t) {
    return t.is_int ? (x > t.ti) : ((double)x > t.td);
}

// Exclusive prefix sum over v[0..n) held one value per thread (n <= blockDim.x == 1024).
// Returns the exclusive prefix of this thread's value; *total gets the sum.  All threads call.
__device__ int block_exclusive_scan(int v, int* total, int* scratch /* [17] LDS */) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int incl = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_up(incl, off);
        if (lane >= off) incl += o;
    }
    if (lane == 63) scratch[wave] = incl;
    __syncthreads();
    if (tid == 0) {
        int run = 0;
        for (int w = 0; w < kFinishThreads / 64; ++w) {
            const int c = scratch[w];
            scratch[w] = run;
            run += c;
        }
        scratch[16] = run;
    }
    __syncthreads();
    const int res = incl - v + scratch[wave];
    *total = scratch[16];
    __syncthreads();
    return res;
}

// mode: 0 = threshold given in td (absolute), 1 = quantile rank k_rank, 2 = mean + kval * std.
// mask / expd / pos are scratch arrays of nb*nb entries (global workspace).
__global__ __launch_bounds__(kFinishThreads) void pattern_finish_kernel(
    const long long* __restrict__ pool, int nb, int mode, long long k_rank, double kval, double t_abs,
    int no_fill, uint8_t* __restrict__ mask, uint8_t* __restrict__ expd, int* __restrict__ pos,
    uint8_t* __restrict__ fl, int* __restrict__ row_ptr, int* __restrict__ col_idx,
    int* __restrict__ col_ptr, int* __restrict__ row_idx, int* __restrict__ bsr_pos,
    int* __restrict__ nnzb_out) {
    const int tid = threadIdx.x;
    const long long n = (long long)nb * nb;
    __shared__ unsigned hist[256];
    __shared__ Thresh th;
    __shared__ unsigned long long sel_prefix;
    __shared__ long long sel_k;
    __shared__ int scan_scratch[17];

    // ---- 1. threshold ------------------------------------------------------------------------
    if (mode == 1) {
        // exact k-th smallest (0-based) by most-significant-byte-first radix selection
        if (tid == 0) {
            sel_prefix = 0ull;
            sel_k = k_rank;
        }
        for (int pass = 7; pass >= 0; --pass) {
            const int shift = pass * 8;
            if (tid < 256) hist[tid] = 0u;
            __syncthreads();
            const unsigned long long prefix = sel_prefix;
            for (long long i = tid; i < n; i += kFinishThreads) {
                const unsigned long long u = (unsigned long long)pool[i] ^ 0x8000000000000000ull;
                const bool match = (pass == 7) || ((u >> (shift + 8)) == (prefix >> (shift + 8)));
                if (match) atomicAdd(&hist[(unsigned)((u >> shift) & 0xFFull)], 1u);
            }
            __syncthreads();
            if (tid == 0) {
                long long k = sel_k;
                int b = 0;
                for (; b < 255; ++b) {
                    const long long c = hist[b];
                    if (k < c) break;
                    k -= c;
                }
                sel_k = k;
                sel_prefix = prefix | ((unsigned long long)b << shift);
            }
            __syncthreads();
        }
        if (tid == 0) {
            th.is_int = 1;
            th.ti = (long long)(sel_prefix ^ 0x8000000000000000ull);
            th.td = (double)th.ti;
        }
    } else if (mode == 2) {
        // sequential fp64 sums in row-major order: this is the definition, not an optimisation target
        if (tid == 0) {
            double sum = 0.0;
            for (long long i = 0; i < n; ++i) sum = sum + (double)pool[i];
            const double mean = sum / (double)n;
            double ss = 0.0;
            for (long long i = 0; i < n; ++i) {
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

    if (no_fill) {
        // SPION-C: keep every block above the threshold
        for (long long i = tid; i < n; i += kFinishThreads) fl[i] = above(pool[i], t) ? 1 : 0;
    } else {
        // ---- 2. successor bits: which of (down, right, diag) equal their maximum ------------------
        for (long long i = tid; i < n; i += kFinishThreads) {
            const int r = (int)(i / nb), c = (int)(i % nb);
            unsigned m = 0u;
            if (r + 1 < nb && c + 1 < nb) {
                const long long dn = pool[i + nb], rt = pool[i + 1], dg = pool[i + nb + 1];
                long long mx = dn > rt ? dn : rt;
                mx = mx > dg ? mx : dg;
                m = (dn == mx ? kDown : 0u) | (rt == mx ? kRight : 0u) | (dg == mx ? kDiag : 0u);
            }
            mask[i] = (uint8_t)m;
            expd[i] = (r == 0 || c == 0) ? 1 : 0;     // seeds: first row and first column
            fl[i] = 0;
        }
        __syncthreads();
        // ---- 3. fill: every move raises r + c, so anti-diagonal s depends only on s-1 and s-2 ----
        // A cell is reached iff an expanded predecessor lists it as a successor; reached cells are
        // expanded in turn (marked or not) and marked iff above the threshold.
        for (int s = 1; s <= 2 * nb - 2; ++s) {
            const int r = tid, c = s - tid;
            if (r < nb && c >= 0 && c < nb) {
                const long long i = (long long)r * nb + c;
                bool reached = false;
                if (r >= 1) reached |= expd[i - nb] && (mask[i - nb] & kDown);
                if (c >= 1) reached |= expd[i - 1] && (mask[i - 1] & kRight);
                if (r >= 1 && c >= 1) reached |= expd[i - nb - 1] && (mask[i - nb - 1] & kDiag);
                if (reached) {
                    expd[i] = 1;
                    if (above(pool[i], t)) fl[i] = 1;
                }
            }
            __syncthreads();
        }
    }
    __syncthreads();
    // ---- 4. forced diagonal ------------------------------------------------------------------------
    if (tid < nb) fl[(long long)tid * nb + tid] = 1;
    __syncthreads();

    // ---- 5. compaction: BSR (rows), then BSC (columns) ---------------------------------------------
    int cnt = 0;
    if (tid < nb)
        for (int c = 0; c < nb; ++c) cnt += fl[(long long)tid * nb + c];
    int total = 0;
    int start = block_exclusive_scan(cnt, &total, scan_scratch);
    if (tid < nb) {
        row_ptr[tid] = start;
        int k = start;
        for (int c = 0; c < nb; ++c) {
            if (fl[(long long)tid * nb + c]) {
                col_idx[k] = c;
                pos[(long long)tid * nb + c] = k;
                ++k;
            }
        }
    }
    if (tid == 0) {
        row_ptr[nb] = total;
        *nnzb_out = total;
    }
    if (col_ptr != nullptr) {
        __syncthreads();
        cnt = 0;
        if (tid < nb)
            for (int r = 0; r < nb; ++r) cnt += fl[(long long)r * nb + tid];
        start = block_exclusive_scan(cnt, &total, scan_scratch);
        if (tid < nb) {
            col_ptr[tid] = start;
            int k = start;
            for (int r = 0; r < nb; ++r) {
                if (fl[(long long)r * nb + tid]) {
                    row_idx[k] = r;
                    bsr_pos[k] = pos[(long long)r * nb + tid];
                    ++k;
                }
            }
        }
        if (tid == 0) col_ptr[nb] = total;
    }
}

// ------------------------------------------------------------------------------------------------
// host launchers
// ------------------------------------------------------------------------------------------------
hipError_t launch_conv_pool(const float* A, int L, int bs, int p, long long* pool, hipStream_t st) {
    const int nb = L / bs;
    const size_t n = (size_t)nb * nb;
    zero_u64_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st>>>(
        reinterpret_cast<unsigned long long*>(pool), n);
    conv_pool_kernel<<<dim3((unsigned)n), dim3(kConvThreads), 0, st>>>(
        A, L, bs, p, reinterpret_cast<unsigned long long*>(pool));
    return hipGetLastError();
}

hipError_t launch_pattern_finish(const long long* pool, int nb, int mode, long long k_rank, double kval,
                                 double t_abs, int no_fill, uint8_t* mask, uint8_t* expd, int* pos,
                                 uint8_t* fl, int* row_ptr, int* col_idx, int* col_ptr, int* row_idx,
                                 int* bsr_pos, int* nnzb, hipStream_t st) {
    pattern_finish_kernel<<<dim3(1), dim3(kFinishThreads), 0, st>>>(
        pool, nb, mode, k_rank, kval, t_abs, no_fill, mask, expd, pos, fl, row_ptr, col_idx, col_ptr,
        row_idx, bsr_pos, nnzb);
    return hipGetLastError();
}

}  // namespace spion
