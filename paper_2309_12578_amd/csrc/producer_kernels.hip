// Producers of the pattern input (both HBM-bound streaming reductions):
//   score_mean_kernel   the attention-score maps of a layer's heads (and batch items) are averaged
//                       into one L x L map before pattern generation (Section 3, "Motivation")
//   frobenius kernels   Eq. 2: distance_i = | ||A^s_{i-1}||_F - ||A^s_i||_F |, the test that ends the
//                       dense-attention phase (Section 4.1)
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "spion_internal.h"

namespace spion {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

// out[i] = (sum over maps m = 0 .. n_maps-1, in that order, of A[m][i]) / n_maps, fp32 arithmetic.
// One thread owns 4 (fp32) or 8 (bf16) consecutive elements; loads of 8 maps are kept in flight.
template <typename T>
__global__ __launch_bounds__(256) void score_mean_kernel(const T* __restrict__ A, int n_maps, size_t n,
                                                         float* __restrict__ out) {
    constexpr int V = 16 / sizeof(T);   // elements per 16-byte load
    const size_t nvec = n / V;
    const float inv = 1.0f / (float)n_maps;
    for (size_t v = (size_t)blockIdx.x * blockDim.x + threadIdx.x; v < nvec; v += (size_t)gridDim.x * blockDim.x) {
        float acc[V];
#pragma unroll
        for (int e = 0; e < V; ++e) acc[e] = 0.f;
        const T* p = A + v * V;
        int m = 0;
        for (; m + 8 <= n_maps; m += 8) {   // 8 maps in flight, added in map order
            if constexpr (sizeof(T) == 4) {
                float4 x[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) x[u] = *reinterpret_cast<const float4*>(p + (size_t)(m + u) * n);
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    acc[0] += x[u].x;
                    acc[1] += x[u].y;
                    acc[2] += x[u].z;
                    acc[3] += x[u].w;
                }
            } else {
                bf16x8_t x[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) x[u] = *reinterpret_cast<const bf16x8_t*>(p + (size_t)(m + u) * n);
#pragma unroll
                for (int u = 0; u < 8; ++u)
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[e] += (float)x[u][e];
            }
        }
        for (; m < n_maps; ++m) {
            if constexpr (sizeof(T) == 4) {
                const float4 x = *reinterpret_cast<const float4*>(p + (size_t)m * n);
                acc[0] += x.x;
                acc[1] += x.y;
                acc[2] += x.z;
                acc[3] += x.w;
            } else {
                const bf16x8_t x = *reinterpret_cast<const bf16x8_t*>(p + (size_t)m * n);
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[e] += (float)x[e];
            }
        }
#pragma unroll
        for (int e = 0; e < V; e += 4)
            *reinterpret_cast<float4*>(out + v * V + e) =
                make_float4(acc[e] * inv, acc[e + 1] * inv, acc[e + 2] * inv, acc[e + 3] * inv);
    }
}

constexpr int kFrobBlocks = 4096, kFrobThreads = 256;

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

// partial[b] = {sum of squares of a, sum of squares of b} over the float4s block b owns (fp64)
__global__ __launch_bounds__(kFrobThreads) void frobenius_partial_kernel(const float* __restrict__ a,
                                                                        const float* __restrict__ b, size_t n,
                                                                        double2* __restrict__ partial) {
    const size_t nvec = n / 4;
    const size_t stride = (size_t)kFrobBlocks * kFrobThreads;
    double sa = 0.0, sb = 0.0;
    auto sq = [](double acc, const float4 x) {
        return acc + ((double)x.x * x.x + (double)x.y * x.y) + ((double)x.z * x.z + (double)x.w * x.w);
    };
    size_t v = (size_t)blockIdx.x * kFrobThreads + threadIdx.x;
    // four float4 of each array in flight per thread
    for (; v + 3 * stride < nvec; v += 4 * stride) {
        float4 x[4], y[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            x[u] = reinterpret_cast<const float4*>(a)[v + u * stride];
            y[u] = reinterpret_cast<const float4*>(b)[v + u * stride];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            sa = sq(sa, x[u]);
            sb = sq(sb, y[u]);
        }
    }
    for (; v < nvec; v += stride) {
        sa = sq(sa, reinterpret_cast<const float4*>(a)[v]);
        sb = sq(sb, reinterpret_cast<const float4*>(b)[v]);
    }
    if (blockIdx.x == 0 && threadIdx.x == 0)   // tail: n not a multiple of 4
        for (size_t i = nvec * 4; i < n; ++i) {
            sa += (double)a[i] * a[i];
            sb += (double)b[i] * b[i];
        }
    __shared__ double2 wsum[kFrobThreads / 64];
    sa = wave_sum_f64(sa);
    sb = wave_sum_f64(sb);
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = make_double2(sa, sb);
    __syncthreads();
    if (threadIdx.x == 0) {
        double ta = 0.0, tb = 0.0;
        for (int w = 0; w < kFrobThreads / 64; ++w) {
            ta += wsum[w].x;
            tb += wsum[w].y;
        }
        partial[blockIdx.x] = make_double2(ta, tb);
    }
}

// out[0] = | sqrt(sum a^2) - sqrt(sum b^2) |, out[1] = ||a||_F, out[2] = ||b||_F; fixed summation order
__global__ __launch_bounds__(kFrobThreads) void frobenius_final_kernel(const double2* __restrict__ partial,
                                                                      double* __restrict__ out) {
    double sa = 0.0, sb = 0.0;
    for (int i = threadIdx.x; i < kFrobBlocks; i += kFrobThreads) {
        sa += partial[i].x;
        sb += partial[i].y;
    }
    __shared__ double2 wsum[kFrobThreads / 64];
    sa = wave_sum_f64(sa);
    sb = wave_sum_f64(sb);
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = make_double2(sa, sb);
    __syncthreads();
    if (threadIdx.x == 0) {
        double ta = 0.0, tb = 0.0;
        for (int w = 0; w < kFrobThreads / 64; ++w) {
            ta += wsum[w].x;
            tb += wsum[w].y;
        }
        const double na = sqrt(ta), nb = sqrt(tb);
        out[0] = fabs(na - nb);
        out[1] = na;
        out[2] = nb;
    }
}

hipError_t launch_score_mean(const void* A, int is_bf16, int n_maps, size_t n, float* out, hipStream_t st) {
    const size_t nvec = n / (is_bf16 ? 8 : 4);
    size_t blocks = (nvec + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    if (is_bf16)
        score_mean_kernel<__bf16><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(static_cast<const __bf16*>(A),
                                                                                 n_maps, n, out);
    else
        score_mean_kernel<float><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(static_cast<const float*>(A),
                                                                               n_maps, n, out);
    return hipGetLastError();
}

size_t frobenius_workspace_bytes() { return (size_t)kFrobBlocks * sizeof(double2); }

hipError_t launch_frobenius_distance(const float* a, const float* b, size_t n, double* out, void* workspace,
                                     hipStream_t st) {
    double2* partial = static_cast<double2*>(workspace);
    frobenius_partial_kernel<<<dim3(kFrobBlocks), dim3(kFrobThreads), 0, st>>>(a, b, n, partial);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    frobenius_final_kernel<<<dim3(1), dim3(kFrobThreads), 0, st>>>(partial, out);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Traffic yardstick: moves n_tiles x 16 KB from src to dst with the access shapes of the attention
// kernels (16 bytes per lane from HBM straight into LDS through the memory pipeline, one wave
// instruction per 1 KB; 16 bytes per lane row stores out).  It reads and writes every byte exactly
// once, so what the hardware traffic counters report for it gives their scale.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void copy_yardstick_kernel(const char* __restrict__ src, char* __restrict__ dst) {
    typedef __attribute__((address_space(3))) void* lds_ptr;
    __shared__ __attribute__((aligned(16))) char tile[16384];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const size_t base = (size_t)blockIdx.x * 16384;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int piece = wave * 4 + k;   // 1 KB pieces
        __builtin_amdgcn_global_load_lds(src + base + piece * 1024 + lane * 16, (lds_ptr)(tile + piece * 1024), 16, 0,
                                         0);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's pieces have landed (it reads only those)
    asm volatile("" ::: "memory");
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int off = (wave * 4 + k) * 1024 + lane * 16;
        *reinterpret_cast<float4*>(dst + base + off) = *reinterpret_cast<const float4*>(tile + off);
    }
}

hipError_t launch_copy_yardstick(const void* src, void* dst, size_t n_tiles, hipStream_t st) {
    copy_yardstick_kernel<<<dim3((unsigned)n_tiles), dim3(256), 0, st>>>(static_cast<const char*>(src),
                                                                        static_cast<char*>(dst));
    return hipGetLastError();
}

}  // namespace spion
