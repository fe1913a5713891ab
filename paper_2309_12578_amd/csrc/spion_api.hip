// C ABI of libspion: argument validation, workspace carving and kernel launches.
// Every entry point validates on the host, enqueues on the caller's stream and returns.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <mutex>

#include "../../include/spion.h"
#include "spion_internal.h"

// Built-in scratch of spion_pattern_static: the pattern workspace (pooled sums, cell bits, the
// transposed mask, positions) for up to SPION_STATIC_MAX_NB^2 blocks.  Every GPU the library runs
// on holds its own copy of this array at its own address until the process ends.  In host code the
// name is only a handle for hipGetSymbolAddress: kernels and copies are given the resolved address.
constexpr size_t kStaticScratchBytes = 5u << 20;   // the workspace of L / block = SPION_STATIC_MAX_NB
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr size_t kAlign = 256;
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};   // per device: address of `scratch` on that device

// Address of `scratch` on the current device, resolved once per device (first call on it) with that
// device current.
int static_scratch(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SPION_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return SPION_ERR_HIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return SPION_OK;
}

size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

bool shape_ok(int32_t L, int32_t block) {
    if (block != 16 && block != 32 && block != 64) return false;
    if (L <= 0 || (L % block) != 0) return false;
    return L / block <= SPION_MAX_NB;
}

// Layout of the pattern workspace for nb*nb = n cells.
struct PatternWs {
    size_t part_off, pool_off, mask_off, expd_off, pos_off, total;
    explicit PatternWs(size_t n) {
        part_off = 0;                                             // one record of 8 int64 per input block
        pool_off = part_off + align_up(8 * n * sizeof(int64_t));
        mask_off = pool_off + align_up(n * sizeof(int64_t));
        expd_off = mask_off + align_up(2 * n);   // cell bits, then the transposed final mask
        pos_off = expd_off + align_up(n);
        total = pos_off + align_up(n * sizeof(int32_t));
    }
};

int attn_params_ok(const spion_attn_params* p, int32_t nnzb) {
    if (p->dtype != SPION_F32 && p->dtype != SPION_BF16) return SPION_ERR_DTYPE;
    if (p->d != 64 || p->B <= 0 || p->H <= 0) return SPION_ERR_SHAPE;
    if (!shape_ok(p->L, p->block)) return SPION_ERR_SHAPE;
    const int64_t nb = p->L / p->block;
    if ((int64_t)p->B * p->H * nb > 0x7fffffffll) return SPION_ERR_SHAPE;   // 1-D grid limit
    if (nnzb < 0 || (int64_t)nnzb > nb * nb) return SPION_ERR_SHAPE;
    if (!(p->scale >= 0.f) || !isfinite(p->scale)) return SPION_ERR_PARAM;
    const uint32_t known = SPION_ATTN_PAPER_DENOM | SPION_ATTN_BWD_QUERY_SIDE_ONLY | SPION_ATTN_BWD_KEY_SIDE_ONLY;
    if (p->flags & ~known) return SPION_ERR_PARAM;
    if ((p->flags & SPION_ATTN_BWD_QUERY_SIDE_ONLY) && (p->flags & SPION_ATTN_BWD_KEY_SIDE_ONLY))
        return SPION_ERR_PARAM;
    return SPION_OK;
}

spion::AttnShape make_shape(const spion_attn_params* p) {
    spion::AttnShape s;
    s.BH = p->B * p->H;
    s.L = p->L;
    s.bs = p->block;
    s.nb = p->L / p->block;
    s.is_bf16 = p->dtype == SPION_BF16;
    s.scale = p->scale > 0.f ? p->scale : 1.0f / sqrtf((float)p->d);
    s.paper_denom = (p->flags & SPION_ATTN_PAPER_DENOM) ? 1 : 0;
    s.bwd_phases = (p->flags & SPION_ATTN_BWD_QUERY_SIDE_ONLY) ? 1
                   : (p->flags & SPION_ATTN_BWD_KEY_SIDE_ONLY) ? 2 : 3;
    return s;
}

}  // namespace

extern "C" {

int spion_version(void) { return 100; }

const char* spion_strerror(int status) {
    switch (status) {
        case SPION_OK: return "ok";
        case SPION_ERR_NULL: return "a required pointer is NULL";
        case SPION_ERR_SHAPE: return "unsupported shape (need d == 64, block in {16,32,64}, L % block == 0)";
        case SPION_ERR_DTYPE: return "unsupported dtype";
        case SPION_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case SPION_ERR_PARAM: return "invalid parameter value";
        case SPION_ERR_INDEX: return "malformed block-sparse index";
        case SPION_ERR_HIP: return "HIP runtime error";
        case SPION_ERR_TOO_LARGE: return "problem exceeds the built-in scratch buffer (L / block > SPION_STATIC_MAX_NB)";
        default: return "unknown status";
    }
}

size_t spion_pattern_workspace_bytes(int32_t L, int32_t block) {
    if (!shape_ok(L, block)) return 0;
    const size_t nb = (size_t)(L / block);
    return PatternWs(nb * nb).total;
}

static int pattern_impl(const float* A_s, const spion_pattern_params* p, uint8_t* fl_out, int32_t* row_ptr,
                        int32_t* col_idx, int32_t* col_ptr, int32_t* row_idx, int32_t* bsr_pos, int32_t* nnzb,
                        int64_t* pool_sum, void* workspace, size_t workspace_bytes, void* hip_stream,
                        bool use_static_scratch) {
    if (!p) return SPION_ERR_NULL;
    const uint32_t known_flags = SPION_PATTERN_NO_FILL | SPION_PATTERN_POOL_ONLY | SPION_PATTERN_FROM_POOL;
    if (p->reserved != 0 || (p->flags & ~known_flags)) return SPION_ERR_PARAM;
    const bool pool_only = (p->flags & SPION_PATTERN_POOL_ONLY) != 0;
    const bool from_pool = (p->flags & SPION_PATTERN_FROM_POOL) != 0;
    if (pool_only && (from_pool || (p->flags & SPION_PATTERN_NO_FILL))) return SPION_ERR_PARAM;
    if (!from_pool && !A_s) return SPION_ERR_NULL;
    if ((pool_only || from_pool) && !pool_sum) return SPION_ERR_NULL;
    if (!pool_only && (!fl_out || !row_ptr || !col_idx || !nnzb)) return SPION_ERR_NULL;
    const bool any_bsc = col_ptr || row_idx || bsr_pos;
    if (any_bsc && !(col_ptr && row_idx && bsr_pos)) return SPION_ERR_NULL;
    if (!shape_ok(p->L, p->block)) return SPION_ERR_SHAPE;
    const int32_t bs = p->block, nb = p->L / bs;
    if (use_static_scratch && nb > SPION_STATIC_MAX_NB) return SPION_ERR_TOO_LARGE;
    if (p->filter < 1 || (p->filter % 2) == 0 || (p->filter - 1) / 2 >= bs) return SPION_ERR_PARAM;
    const int64_t n = (int64_t)nb * nb;
    int mode = 0;
    long long k_rank = 0;
    double kval = 0.0, t_abs = 0.0;
    switch (p->thresh_mode) {
        case SPION_T_ABS: {
            if (!isfinite(p->thresh_value)) return SPION_ERR_PARAM;
            const double cells = (double)bs * (double)bs;
            const double scaled = p->thresh_value * cells;
            t_abs = scaled * 1099511627776.0;   // pool_sum units: block^2 * 2^40
            mode = 0;
            break;
        }
        case SPION_T_QUANTILE: {
            if (!(p->thresh_value >= 0.0 && p->thresh_value <= 1.0)) return SPION_ERR_PARAM;
            k_rank = (long long)floor(p->thresh_value * (double)(n - 1));
            if (k_rank < 0) k_rank = 0;
            if (k_rank > n - 1) k_rank = n - 1;
            mode = 1;
            break;
        }
        case SPION_T_MEAN_KSTD:
            if (!isfinite(p->thresh_value)) return SPION_ERR_PARAM;
            kval = p->thresh_value;
            mode = 2;
            break;
        default: return SPION_ERR_PARAM;
    }
    const PatternWs ws((size_t)n);
    if (use_static_scratch) {
        // every argument has passed validation; only now is the device touched
        const int rc = static_scratch(&workspace);
        if (rc != SPION_OK) return rc;
        workspace_bytes = kStaticScratchBytes;
    }
    if (!workspace || ((uintptr_t)workspace % kAlign) != 0 || workspace_bytes < ws.total)
        return SPION_ERR_WORKSPACE;
    char* w = static_cast<char*>(workspace);
    long long* pool = pool_sum ? reinterpret_cast<long long*>(pool_sum)
                               : reinterpret_cast<long long*>(w + ws.pool_off);
    long long* part = reinterpret_cast<long long*>(w + ws.part_off);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (!from_pool && spion::launch_conv_pool(A_s, p->L, bs, (p->filter - 1) / 2, part, st) != hipSuccess)
        return SPION_ERR_HIP;
    if (pool_only)
        return spion::launch_pool_gather(part, nb, pool, st) == hipSuccess ? SPION_OK : SPION_ERR_HIP;
    if (spion::launch_pattern_finish(from_pool ? nullptr : part, pool, nb, mode, k_rank, kval, t_abs,
                                     (p->flags & SPION_PATTERN_NO_FILL) ? 1 : 0,
                                     reinterpret_cast<uint8_t*>(w + ws.mask_off),
                                     reinterpret_cast<uint8_t*>(w + ws.expd_off),
                                     reinterpret_cast<int*>(w + ws.pos_off), fl_out, row_ptr, col_idx,
                                     col_ptr, row_idx, bsr_pos, nnzb, st) != hipSuccess)
        return SPION_ERR_HIP;
    return SPION_OK;
}

int spion_pattern(const float* A_s, const spion_pattern_params* p, uint8_t* fl_out, int32_t* row_ptr,
                  int32_t* col_idx, int32_t* col_ptr, int32_t* row_idx, int32_t* bsr_pos, int32_t* nnzb,
                  int64_t* pool_sum, void* workspace, size_t workspace_bytes, void* hip_stream) {
    return pattern_impl(A_s, p, fl_out, row_ptr, col_idx, col_ptr, row_idx, bsr_pos, nnzb, pool_sum, workspace,
                        workspace_bytes, hip_stream, false);
}

int spion_pattern_static(const float* A_s, const spion_pattern_params* p, uint8_t* fl_out, int32_t* row_ptr,
                         int32_t* col_idx, int32_t* col_ptr, int32_t* row_idx, int32_t* bsr_pos,
                         int32_t* nnzb, int64_t* pool_sum, void* hip_stream) {
    return pattern_impl(A_s, p, fl_out, row_ptr, col_idx, col_ptr, row_idx, bsr_pos, nnzb, pool_sum, nullptr, 0,
                        hip_stream, true);
}

int spion_score_mean(const void* A_maps, int32_t n_maps, int32_t L, int32_t dtype, float* A_s,
                     void* hip_stream) {
    if (!A_maps || !A_s) return SPION_ERR_NULL;
    if (dtype != SPION_F32 && dtype != SPION_BF16) return SPION_ERR_DTYPE;
    if (n_maps <= 0 || L <= 0 || (L % 8) != 0) return SPION_ERR_SHAPE;
    if (spion::launch_score_mean(A_maps, dtype == SPION_BF16, n_maps, (size_t)L * L, A_s,
                                 static_cast<hipStream_t>(hip_stream)) != hipSuccess)
        return SPION_ERR_HIP;
    return SPION_OK;
}

size_t spion_frobenius_workspace_bytes(void) { return align_up(spion::frobenius_workspace_bytes()); }

int spion_frobenius_distance(const float* A_prev, const float* A_cur, int64_t n, double* out,
                             void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!A_prev || !A_cur || !out) return SPION_ERR_NULL;
    if (n <= 0) return SPION_ERR_SHAPE;
    if (((uintptr_t)A_prev % 16) != 0 || ((uintptr_t)A_cur % 16) != 0) return SPION_ERR_PARAM;
    if (!workspace || ((uintptr_t)workspace % kAlign) != 0 ||
        workspace_bytes < spion_frobenius_workspace_bytes())
        return SPION_ERR_WORKSPACE;
    if (spion::launch_frobenius_distance(A_prev, A_cur, (size_t)n, out, workspace,
                                         static_cast<hipStream_t>(hip_stream)) != hipSuccess)
        return SPION_ERR_HIP;
    return SPION_OK;
}

int spion_copy_yardstick(const void* src, void* dst, size_t n_bytes, void* hip_stream) {
    if (!src || !dst) return SPION_ERR_NULL;
    if (n_bytes == 0 || (n_bytes % 16384) != 0 || n_bytes / 16384 > 0x7fffffffull) return SPION_ERR_SHAPE;
    if (((uintptr_t)src % 16) != 0 || ((uintptr_t)dst % 16) != 0) return SPION_ERR_PARAM;
    if (spion::launch_copy_yardstick(src, dst, n_bytes / 16384, static_cast<hipStream_t>(hip_stream)) != hipSuccess)
        return SPION_ERR_HIP;
    return SPION_OK;
}

size_t spion_attn_workspace_bytes(const spion_attn_params* p, int32_t nnzb, int32_t is_bwd) {
    if (!p || attn_params_ok(p, nnzb) != SPION_OK) return (size_t)-1;
    if (!is_bwd) return 0;
    return spion::attn_bwd_workspace_bytes(p->B * p->H, p->L, p->block, p->L / p->block, nnzb);
}

int spion_index_check(const int32_t* row_ptr, const int32_t* col_idx, const int32_t* col_ptr,
                      const int32_t* row_idx, const int32_t* bsr_pos, int32_t nb, int32_t nnzb,
                      int32_t* status, void* hip_stream) {
    if (!row_ptr || !col_idx || !status) return SPION_ERR_NULL;
    const bool any_bsc = col_ptr || row_idx || bsr_pos;
    if (any_bsc && !(col_ptr && row_idx && bsr_pos)) return SPION_ERR_NULL;
    if (nb <= 0 || nb > SPION_MAX_NB || nnzb < 0 || (int64_t)nnzb > (int64_t)nb * nb) return SPION_ERR_SHAPE;
    if (spion::launch_index_check(row_ptr, col_idx, col_ptr, row_idx, bsr_pos, nb, nnzb, SPION_ERR_INDEX,
                                  status, static_cast<hipStream_t>(hip_stream)) != hipSuccess)
        return SPION_ERR_HIP;
    return SPION_OK;
}

int spion_attn_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE,
                   const int32_t* row_ptr, const int32_t* col_idx, int32_t nnzb,
                   const spion_attn_params* p, void* workspace, size_t workspace_bytes,
                   void* hip_stream) {
    (void)workspace;
    (void)workspace_bytes;
    if (!Q || !K || !V || !O || !LSE || !row_ptr || !col_idx || !p) return SPION_ERR_NULL;
    const int rc = attn_params_ok(p, nnzb);
    if (rc != SPION_OK) return rc;
    const spion::AttnShape s = make_shape(p);
    if (spion::launch_attn_fwd(s, Q, K, V, O, LSE, row_ptr, col_idx,
                               static_cast<hipStream_t>(hip_stream)) != hipSuccess)
        return SPION_ERR_HIP;
    return SPION_OK;
}

int spion_attn_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                   const float* LSE, void* dQ, void* dK, void* dV, const int32_t* row_ptr,
                   const int32_t* col_idx, const int32_t* col_ptr, const int32_t* row_idx,
                   const int32_t* bsr_pos, int32_t nnzb, const spion_attn_params* p, void* workspace,
                   size_t workspace_bytes, void* hip_stream) {
    if (!Q || !K || !V || !O || !dO || !LSE || !dQ || !dK || !dV || !row_ptr || !col_idx || !col_ptr ||
        !row_idx || !bsr_pos || !p)
        return SPION_ERR_NULL;
    const int rc = attn_params_ok(p, nnzb);
    if (rc != SPION_OK) return rc;
    if (!spion::attn_bwd_grids_fit(p->B * p->H, p->L, p->block, p->L / p->block, nnzb)) return SPION_ERR_SHAPE;
    const size_t need = spion_attn_workspace_bytes(p, nnzb, 1);
    if (!workspace || ((uintptr_t)workspace % kAlign) != 0 || workspace_bytes < need)
        return SPION_ERR_WORKSPACE;
    const spion::AttnShape s = make_shape(p);
    if (spion::launch_attn_bwd(s, Q, K, V, O, dO, LSE, dQ, dK, dV, row_ptr, col_idx, col_ptr, row_idx,
                               nnzb, workspace, static_cast<hipStream_t>(hip_stream)) != hipSuccess)
        return SPION_ERR_HIP;
    return SPION_OK;
}

}  // extern "C"
