// Shared declarations of the HIP sources of the SCFA library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <atomic>

#include "scfa.h"

namespace scfa {

// ---- error plumbing ---------------------------------------------------------
extern thread_local int g_last_hip_error;

inline int hip_fail(hipError_t e)
{
    g_last_hip_error = (int)e;
    return SCFA_EHIP;
}

#define SCFA_HIP_TRY(expr)                                 \
    do {                                                   \
        hipError_t _e = (expr);                            \
        if (_e != hipSuccess) return ::scfa::hip_fail(_e); \
    } while (0)

// A kernel that takes more than 64 KB of dynamic LDS has to be told so once on every device it
// runs on.  `done` (one per kernel instantiation) remembers the devices already prepared, one
// bit each; the current device is the one the caller's stream belongs to.
inline int allow_dynamic_lds(const void* kernel, int bytes, std::atomic<unsigned long long>& done)
{
    int dev = 0;
    SCFA_HIP_TRY(hipGetDevice(&dev));
    const unsigned long long bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return SCFA_OK;
    SCFA_HIP_TRY(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
    done.fetch_or(bit, std::memory_order_release);
    return SCFA_OK;
}

// ---- profiling hooks (scfa_prof_*) -----------------------------------------
struct ProfScope {
    int kid;
    hipStream_t stream;
    int slot;
    ProfScope(int kernel_id, hipStream_t s);
    ~ProfScope();
};

// ---- work list layout (see scfa_block_ranges) -------------------------------
constexpr int WORK_STRIDE = SCFA_WORK_STRIDE;

// forward / dQ items
constexpr int W_QBEGIN = 0, W_QCOUNT = 1, W_KBEGIN = 2, W_KCOUNT = 3, W_KNOMASK = 4, W_BUCKET = 5, W_NBUCKETS = 6;
// backward (key-major) items
constexpr int BW_KBEGIN = 0, BW_KCOUNT = 1, BW_QBEGIN = 2, BW_QCOUNT = 3, BW_QMASKED = 4;

// ---- sort keys ------------------------------------------------------------------
// The attention kernels identify a sorted row by its sort key, bucket << 24 | original position
// (scfa_sort_by_bucket's sort_key_out; a compacted index vector of QK-dropping is its own key,
// the one bucket having id 0).  Keys increase along the sorted rows of a segment, and "same
// bucket, position <= p" is one unsigned range test: (key - (bucket << 24)) <= p.
constexpr uint32_t KEY_POS_BITS = 24;
constexpr uint32_t KEY_POS_MASK = (1u << KEY_POS_BITS) - 1u;
constexpr uint32_t KEY_PAST_END = 0xffffffffu;   // rows past the end of a ragged tile: match no range
constexpr uint32_t KEY_NEVER = 0xfffffffeu;      // lower end of the range of a row that may match nothing

// ---- tile configuration -------------------------------------------------------
constexpr int FWD_TILE_M = 128;  // query rows per workgroup (4 waves x 32)
constexpr int FWD_TILE_N = 64;   // keys per inner step
constexpr int BWD_TILE_N = 128;  // key rows per workgroup in the dK/dV kernel (4 waves x 32)
constexpr int BWD_TILE_M = 64;   // query rows per inner step of the dK/dV kernel
constexpr int F32_TILE_M = 64;   // fp32 path: one thread per query row
constexpr int F32_TILE_N = 32;

// ---- kernel launchers (defined in the .hip files) ---------------------------
int launch_sort_by_bucket(int n_problems, const int32_t* bucket0, const int32_t* bucket1, int S, int T, int nb,
                          int32_t* idx0, int32_t* sorted0, int32_t* off0, uint32_t* key0, int32_t* idx1,
                          int32_t* sorted1, int32_t* off1, uint32_t* key1, void* ws, size_t ws_bytes, hipStream_t st);
int launch_count_invalid_buckets(const int32_t* bucket, long long n, int nb, int32_t* counter, hipStream_t st);
int launch_sort_by_bucket_static(const int32_t* bucket, int S, int T, int nb, int32_t* idx, int32_t* sorted,
                                 int32_t* off, uint32_t* key, hipStream_t st);
int launch_compact_keep(int n_problems, const uint8_t* keep0, const uint8_t* keep1, int S, int T, int32_t* idx0,
                        int32_t* count0, int32_t* idx1, int32_t* count1, void* ws, size_t ws_bytes, hipStream_t st);
size_t sort_workspace_bytes(int n_problems, int S, int T, int nb);
int launch_lsh_buckets(int n_problems, const void* x0, const void* x1, const float* R, int S, int H, int T, int d,
                       int nb, bool bf16, int32_t* out0, int32_t* out1, hipStream_t st);
int launch_gather_rows(int n_tensors, const void* const* x, const int32_t* const* idx, const int32_t* const* count,
                       const float* scale, void* const* out, int S, int T, int row_bytes, int mode, hipStream_t st);
int launch_block_ranges(int variant, const int32_t* q_idx, const int32_t* k_idx,
                        const int32_t* q_off, const int32_t* k_off, int S, int T, int nb,
                        int fwd_m, int fwd_n, int bwd_n, int bwd_m, int n_fwd, int n_bwd, int strict,
                        int32_t* fwd_work, int32_t* bwd_work, int64_t* counters, hipStream_t st);
int launch_zero_rows(const int32_t* idx, const int32_t* count, int S, int T, int row_bytes,
                     void* out0, void* out1, float* vec, float vec_value, hipStream_t st);
int launch_attn_fwd_f32(const float* q, const float* k, const float* v, const uint32_t* q_key,
                        const uint32_t* k_key, const int32_t* work, int n_work, int S, int T, int d,
                        float tau, int strict, float* o, float* lse, hipStream_t st);
int launch_attn_fwd_bf16(const void* q, const void* k, const void* v, const uint32_t* q_key,
                         const uint32_t* k_key, const int32_t* work, int n_work, int S, int T, int d,
                         float tau, int strict, void* o, float* lse, void* o_f16, const int32_t* n_keep_q,
                         hipStream_t st);   // n_keep_q: QK-dropping (the kernel writes the dropped rows), else null
int launch_bwd_prep_bf16(const void* o, const void* o_f16, const float* lse, const void* d_o, const uint32_t* q_key,
                         const int32_t* n_q,
                         int S, int T, int d, float tau, void* do_perm, float* delta_perm, float* lse_perm,
                         void* aux_perm, uint32_t* amax, float* inv_scale, hipStream_t st);
int launch_attn_bwd_dkdv_bf16(const void* q, const void* k, const void* v, const void* do_perm,
                              const void* aux_perm, const float* inv_scale,
                              const uint32_t* q_key, const uint32_t* k_key, const int32_t* bwd_work, int n_bwd,
                              int S, int T, int d, float tau, int strict, float* dk, float* dv, const int32_t* n_keep_k,
                              hipStream_t st);
int launch_attn_bwd_dq_bf16(const void* q, const void* k, const void* v, const void* do_perm,
                            const float* lse_perm, const float* delta_perm, const float* inv_scale,
                            const uint32_t* q_key, const uint32_t* k_key, const int32_t* fwd_work, int n_fwd,
                            int S, int T, int d, float tau, int strict, float* dq, const int32_t* n_keep_q, hipStream_t st);

int occupancy_attn_fwd_bf16(int d, int* out);
int occupancy_attn_bwd_dkdv_bf16(int d, int* out);
int occupancy_attn_bwd_dq_bf16(int d, int* out);

}  // namespace scfa
