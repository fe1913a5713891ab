// Internal launcher declarations shared by the translation units of libspion (not installed).
#ifndef SPION_INTERNAL_H_
#define SPION_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace spion {

// pattern_kernels.hip
// part: one record of 8 int64 per input block (nb * nb records), written by launch_conv_pool;
// launch_pool_gather / launch_pattern_finish add them up into pool[nb * nb].  launch_pattern_finish
// with part == nullptr starts from a given pool[].
hipError_t launch_conv_pool(const float* A, int L, int bs, int p, long long* part, hipStream_t st);
hipError_t launch_pool_gather(const long long* part, int nb, long long* pool, hipStream_t st);
hipError_t launch_pattern_finish(const long long* part, long long* pool, int nb, int mode, long long k_rank,
                                 double kval, double t_abs, int no_fill, uint8_t* mask, uint8_t* expd, int* pos,
                                 uint8_t* fl, int* row_ptr, int* col_idx, int* col_ptr, int* row_idx,
                                 int* bsr_pos, int* nnzb, hipStream_t st);

// producer_kernels.hip
hipError_t launch_index_check(const int* row_ptr, const int* col_idx, const int* col_ptr, const int* row_idx,
                              const int* bsr_pos, int nb, int nnzb, int err_code, int* status, hipStream_t st);
hipError_t launch_score_mean(const void* A, int is_bf16, int n_maps, size_t n, float* out, hipStream_t st);
hipError_t launch_copy_yardstick(const void* src, void* dst, size_t n_tiles, hipStream_t st);
size_t frobenius_workspace_bytes();
hipError_t launch_frobenius_distance(const float* a, const float* b, size_t n, double* out, void* workspace,
                                     hipStream_t st);

// attn_kernels.hip
struct AttnShape {
    int BH, L, bs, nb;
    int is_bf16;
    float scale;        // resolved score scale (> 0)
    int paper_denom;    // Algorithm 6's extra denominator term
    int bwd_phases;     // bit 0: query-side kernel (delta, dQ); bit 1: key-side kernel (dK, dV)
};

hipError_t launch_attn_fwd(const AttnShape& s, const void* Q, const void* K, const void* V, void* O,
                           float* LSE, const int* row_ptr, const int* col_idx, hipStream_t st);
hipError_t launch_attn_bwd(const AttnShape& s, const void* Q, const void* K, const void* V,
                           const void* O, const void* dO, const float* LSE, void* dQ, void* dK,
                           void* dV, const int* row_ptr, const int* col_idx, const int* col_ptr,
                           const int* row_idx, int nnzb, void* workspace, hipStream_t st);

// Carving of the backward workspace: delta = rowsum(dO .* O) per query, the key-side work list, and
// fp32 partial dK / dV tiles for block columns that are cut into several chunks.
struct BwdWorkspace {
    int w_max, n_slots, split_max;
    size_t delta_off, sched_off, split_off, partial_off, total;
    BwdWorkspace(int BH, int L, int bs, int nb, int nnzb);
};
size_t attn_bwd_workspace_bytes(int BH, int L, int bs, int nb, int nnzb);
// false when a backward launch for this shape would need more workgroups than a 1-D grid can hold
bool attn_bwd_grids_fit(int BH, int L, int bs, int nb, int nnzb);

// attn_bf16_kernels.hip: tuned bf16 forward, BS in {32, 64}
template <int BS>
hipError_t fwd_bf16(const AttnShape& s, const void* Q, const void* K, const void* V, void* O, float* LSE,
                    const int* row_ptr, const int* col_idx, hipStream_t st);

// attn_bwd_bf16_kernels.hip: tuned bf16 backward, BS in {32, 64}; both sides in one launch plus the
// reduction of the partial tiles of split block columns
template <int BS>
hipError_t bwd_bf16(const AttnShape& s, const void* Q, const void* K, const void* V, const void* O,
                    const void* dO, const float* LSE, void* dQ, void* dK, void* dV, const int* row_ptr,
                    const int* col_idx, const int* col_ptr, const int* row_idx, int nnzb, int w_max,
                    int split_max, int n_slots, float* partial, hipStream_t st);

}  // namespace spion
#endif
