// C ABI of the SCFA library: argument checks, workspace carving, kernel sequencing,
// and the event-based per-kernel timers.  See include/scfa.h for the contract.
#include "scfa_common.hpp"

#include <math.h>

#include <mutex>
#include <vector>

namespace scfa {

thread_local int g_last_hip_error = 0;

// ---- per-kernel timers --------------------------------------------------------
namespace {
struct ProfRec { int kid; hipEvent_t a, b; };
std::mutex g_prof_mu;
bool g_prof_on = false;
std::vector<ProfRec> g_prof_recs;      // records of the current measurement
std::vector<hipEvent_t> g_prof_pool;   // recycled events
constexpr size_t PROF_MAX_RECS = 1 << 16;

hipEvent_t prof_get_event()
{
    if (!g_prof_pool.empty()) {
        hipEvent_t e = g_prof_pool.back();
        g_prof_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}
}  // namespace

ProfScope::ProfScope(int kernel_id, hipStream_t s) : kid(kernel_id), stream(s), slot(-1)
{
    if (!g_prof_on || kernel_id < 0) return;   // a negative id: a launch that must not create events
    std::lock_guard<std::mutex> lk(g_prof_mu);
    if (g_prof_recs.size() >= PROF_MAX_RECS) return;
    ProfRec r{kernel_id, prof_get_event(), prof_get_event()};
    if (!r.a || !r.b) return;
    (void)hipEventRecord(r.a, s);
    g_prof_recs.push_back(r);
    slot = (int)g_prof_recs.size() - 1;
}

ProfScope::~ProfScope()
{
    if (slot < 0) return;
    std::lock_guard<std::mutex> lk(g_prof_mu);
    if ((size_t)slot < g_prof_recs.size()) (void)hipEventRecord(g_prof_recs[slot].b, stream);
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

static int check_attn_common(const void* q, const void* k, const void* v, const uint32_t* q_key,
                             const uint32_t* k_key, const int32_t* work, int n_work, int B, int H, int T,
                             int d, int dtype, float sm_scale, int flags)
{
    if (!q || !k || !v || !q_key || !k_key || !work) return SCFA_EINVAL;
    if (B <= 0 || H <= 0 || T <= 0 || n_work <= 0) return SCFA_EINVAL;
    if (T > SCFA_MAX_T) return SCFA_EUNSUPPORTED;   // positions take the low 24 bits of a sort key
    if ((long long)T * d * 4 > 0x7fffffffLL) return SCFA_EUNSUPPORTED;   // byte offsets inside a segment are 32-bit
    if (!(sm_scale > 0.f) || !isfinite(sm_scale)) return SCFA_EINVAL;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v)) return SCFA_EINVAL;
    if ((flags & ~SCFA_FLAG_STRICT_CAUSAL) != 0) return SCFA_EUNSUPPORTED;
    if (dtype != SCFA_BF16 && dtype != SCFA_F32) return SCFA_EUNSUPPORTED;
    if (d != 64 && d != 128) return SCFA_EUNSUPPORTED;
    if ((long long)B * H * (long long)n_work > 0x7fffffffLL) return SCFA_EUNSUPPORTED;
    if ((long long)B * H > 65535) return SCFA_EUNSUPPORTED;
    return SCFA_OK;
}

static int attn_fwd_impl(const void* q, const void* k, const void* v, const uint32_t* q_key,
                         const uint32_t* k_key, const int32_t* n_q, bool qkdrop, const int32_t* work,
                         int n_work, int B, int H, int T, int d, int dtype, float sm_scale, int flags,
                         void* o, float* lse, void* o_f16, hipStream_t st)
{
    int rc = check_attn_common(q, k, v, q_key, k_key, work, n_work, B, H, T, d, dtype, sm_scale, flags);
    if (rc != SCFA_OK) return rc;
    if (!o || !lse || !aligned16(o)) return SCFA_EINVAL;
    if (qkdrop && !n_q) return SCFA_EINVAL;
    if (o_f16 && (dtype != SCFA_BF16 || !aligned16(o_f16))) return SCFA_EINVAL;
    const int S = B * H;
    const int esize = dtype == SCFA_BF16 ? 2 : 4;
    if (dtype == SCFA_F32) {
        if (qkdrop) {   // rows of dropped queries: zeros, LSE = -inf
            rc = launch_zero_rows(reinterpret_cast<const int32_t*>(q_key), n_q, S, T, d * esize, o, nullptr, lse, -INFINITY, st);
            if (rc != SCFA_OK) return rc;
        }
        return launch_attn_fwd_f32((const float*)q, (const float*)k, (const float*)v, q_key, k_key, work,
                                   n_work, S, T, d, sm_scale, flags & SCFA_FLAG_STRICT_CAUSAL, (float*)o, lse, st);
    }
    // bf16: the forward kernel writes the rows of dropped queries itself
    return launch_attn_fwd_bf16(q, k, v, q_key, k_key, work, n_work, S, T, d, sm_scale, flags & SCFA_FLAG_STRICT_CAUSAL, o,
                                lse, o_f16, qkdrop ? n_q : nullptr, st);
}

static int attn_bwd_impl(const void* q, const void* k, const void* v, const uint32_t* q_key,
                         const uint32_t* k_key, const int32_t* n_q, const int32_t* n_k, bool qkdrop,
                         const int32_t* fwd_work, int n_fwd, const int32_t* bwd_work, int n_bwd,
                         const void* o, const void* o_f16, const float* lse, const void* d_o, int B, int H,
                         int T, int d, int dtype, float sm_scale, int flags, float* dq, float* dk, float* dv,
                         void* ws, size_t ws_bytes, hipStream_t st)
{
    int rc = check_attn_common(q, k, v, q_key, k_key, fwd_work, n_fwd, B, H, T, d, dtype, sm_scale, flags);
    if (rc != SCFA_OK) return rc;
    if (!bwd_work || n_bwd <= 0 || (!o && !o_f16) || !lse || !d_o || !dq || !dk || !dv || !ws) return SCFA_EINVAL;
    if (!aligned16(o) || !aligned16(o_f16) || !aligned16(d_o) || !aligned16(dq) || !aligned16(dk) || !aligned16(dv)) return SCFA_EINVAL;
    if ((reinterpret_cast<uintptr_t>(ws) & 255u) != 0) return SCFA_EINVAL;
    if (qkdrop && (!n_q || !n_k)) return SCFA_EINVAL;
    if (dtype != SCFA_BF16) return SCFA_EUNSUPPORTED;
    if ((long long)B * H * (long long)n_bwd > 0x7fffffffLL) return SCFA_EUNSUPPORTED;
    const int S = B * H;
    if (ws_bytes < scfa_attn_bwd_workspace_bytes(S, T, d, dtype)) return SCFA_EWORKSPACE;

    unsigned char* w = reinterpret_cast<unsigned char*>(ws);
    void* do_perm = w;
    w += align_up((size_t)S * T * d * 2, 256);
    float* delta_perm = reinterpret_cast<float*>(w);
    w += align_up((size_t)S * T * 4, 256);
    float* lse_perm = reinterpret_cast<float*>(w);
    w += align_up((size_t)S * T * 4, 256);
    void* aux_perm = w;                         // [S,T,8] fp16: pieces of LSE log2 e and D
    w += align_up((size_t)S * T * 16, 256);
    uint32_t* amax = reinterpret_cast<uint32_t*>(w);   // [S,64] partial maxima of |dO|
    w += align_up((size_t)S * 64 * 4, 256);
    float* inv_scale = reinterpret_cast<float*>(w);

    rc = launch_bwd_prep_bf16(o, o_f16, lse, d_o, q_key, qkdrop ? n_q : nullptr, S, T, d, sm_scale, do_perm, delta_perm, lse_perm, aux_perm, amax, inv_scale, st);
    if (rc != SCFA_OK) return rc;
    // The rows of dropped tokens (QK-dropping) are zeroed by the two gradient kernels themselves, next to their own stores:
    // as launches of their own in front of the pre-pass, half a gigabyte of fresh zeros on its way out of the caches halved
    // the pace of the pre-pass's streaming reads, and anywhere on this stream they would run with nothing beside them.
    rc = launch_attn_bwd_dkdv_bf16(q, k, v, do_perm, aux_perm, inv_scale, q_key, k_key, bwd_work, n_bwd, S, T, d,
                                   sm_scale, flags & SCFA_FLAG_STRICT_CAUSAL, dk, dv, qkdrop ? n_k : nullptr, st);
    if (rc != SCFA_OK) return rc;
    return launch_attn_bwd_dq_bf16(q, k, v, do_perm, lse_perm, delta_perm, inv_scale, q_key, k_key, fwd_work, n_fwd,
                                   S, T, d, sm_scale, flags & SCFA_FLAG_STRICT_CAUSAL, dq, qkdrop ? n_q : nullptr, st);
}

}  // namespace scfa

using namespace scfa;

extern "C" {

int scfa_version(void) { return 100; }

int scfa_last_hip_error(void) { return g_last_hip_error; }

const char* scfa_error_string(int code)
{
    switch (code) {
        case SCFA_OK: return "ok";
        case SCFA_EINVAL: return "invalid argument";
        case SCFA_EUNSUPPORTED: return "unsupported dtype, head dimension, bucket count, tile size or flag";
        case SCFA_EWORKSPACE: return "workspace too small";
        case SCFA_EHIP: return "HIP runtime error";
        default: return "unknown error";
    }
}

size_t scfa_sort_workspace_bytes(int S, int T, int nb)
{
    if (S <= 0 || T <= 0 || nb <= 0 || S > 0x3fffffff) return 0;
    const size_t one = sort_workspace_bytes(1, S, T, nb < 2 ? 2 : nb), two = sort_workspace_bytes(2, S, T, nb < 2 ? 2 : nb);
    return align_up(one > two ? one : two, 256);
}

int scfa_sort_by_bucket(const int32_t* bucket, int S, int T, int nb, int32_t* idx_out,
                        int32_t* bucket_sorted_out, int32_t* bucket_off_out, uint32_t* sort_key_out,
                        void* ws, size_t ws_bytes, void* stream)
{
    if (!bucket || !idx_out || !bucket_off_out || S <= 0 || T <= 0 || nb <= 0) return SCFA_EINVAL;
    if (nb > SCFA_MAX_BUCKETS || S > 0x7fffffff / 1) return SCFA_EUNSUPPORTED;
    if (sort_key_out && T > SCFA_MAX_T) return SCFA_EUNSUPPORTED;
    return launch_sort_by_bucket(1, bucket, nullptr, S, T, nb, idx_out, bucket_sorted_out, bucket_off_out, sort_key_out,
                                 nullptr, nullptr, nullptr, nullptr, ws, ws_bytes, (hipStream_t)stream);
}

int scfa_count_invalid_buckets(const int32_t* bucket, long long n, int nb, int32_t* n_invalid_out, void* stream)
{
    if (!bucket || !n_invalid_out || n < 0 || nb <= 0) return SCFA_EINVAL;
    if (nb > SCFA_MAX_BUCKETS) return SCFA_EUNSUPPORTED;
    return launch_count_invalid_buckets(bucket, n, nb, n_invalid_out, (hipStream_t)stream);
}

int scfa_sort_by_bucket_static(const int32_t* bucket, int S, int T, int nb, int32_t* idx_out,
                               int32_t* bucket_sorted_out, int32_t* bucket_off_out, uint32_t* sort_key_out,
                               void* stream)
{
    if (!bucket || !idx_out || !bucket_off_out || S <= 0 || T <= 0 || nb <= 0) return SCFA_EINVAL;
    if (nb > SCFA_MAX_BUCKETS) return SCFA_EUNSUPPORTED;
    if (sort_key_out && T > SCFA_MAX_T) return SCFA_EUNSUPPORTED;
    return launch_sort_by_bucket_static(bucket, S, T, nb, idx_out, bucket_sorted_out, bucket_off_out, sort_key_out,
                                        (hipStream_t)stream);
}

int scfa_sort_by_bucket_pair(const int32_t* bucket_q, const int32_t* bucket_k, int S, int T, int nb,
                             int32_t* q_idx_out, int32_t* q_sorted_out, int32_t* q_off_out, uint32_t* q_sort_key_out,
                             int32_t* k_idx_out, int32_t* k_sorted_out, int32_t* k_off_out, uint32_t* k_sort_key_out,
                             void* ws, size_t ws_bytes, void* stream)
{
    if (!bucket_q || !bucket_k || !q_idx_out || !q_off_out || !k_idx_out || !k_off_out || S <= 0 || T <= 0 || nb <= 0)
        return SCFA_EINVAL;
    if (nb > SCFA_MAX_BUCKETS || S > 0x3fffffff) return SCFA_EUNSUPPORTED;
    if ((q_sort_key_out || k_sort_key_out) && T > SCFA_MAX_T) return SCFA_EUNSUPPORTED;
    return launch_sort_by_bucket(2, bucket_q, bucket_k, S, T, nb, q_idx_out, q_sorted_out, q_off_out, q_sort_key_out,
                                 k_idx_out, k_sorted_out, k_off_out, k_sort_key_out, ws, ws_bytes, (hipStream_t)stream);
}

int scfa_compact_keep(const uint8_t* keep, int S, int T, int32_t* idx_out, int32_t* count_out, void* ws,
                      size_t ws_bytes, void* stream)
{
    if (!keep || !idx_out || !count_out || S <= 0 || T <= 0) return SCFA_EINVAL;
    return launch_compact_keep(1, keep, nullptr, S, T, idx_out, count_out, nullptr, nullptr, ws, ws_bytes,
                               (hipStream_t)stream);
}

int scfa_compact_keep_pair(const uint8_t* keep_q, const uint8_t* keep_k, int S, int T, int32_t* q_idx_out,
                           int32_t* n_q_out, int32_t* k_idx_out, int32_t* n_k_out, void* ws, size_t ws_bytes,
                           void* stream)
{
    if (!keep_q || !keep_k || !q_idx_out || !n_q_out || !k_idx_out || !n_k_out || S <= 0 || T <= 0) return SCFA_EINVAL;
    if (S > 0x3fffffff) return SCFA_EUNSUPPORTED;
    return launch_compact_keep(2, keep_q, keep_k, S, T, q_idx_out, n_q_out, k_idx_out, n_k_out, ws, ws_bytes,
                               (hipStream_t)stream);
}

int scfa_lsh_buckets(const void* x_q, const void* x_k, const float* R, int S, int H, int T, int d, int nb, int dtype,
                     int32_t* bucket_q_out, int32_t* bucket_k_out, void* stream)
{
    if (!x_q || !R || !bucket_q_out || S <= 0 || H <= 0 || T <= 0 || nb <= 0) return SCFA_EINVAL;
    if ((x_k == nullptr) != (bucket_k_out == nullptr)) return SCFA_EINVAL;
    if (S % H != 0 || (nb & 1) != 0) return SCFA_EINVAL;
    if (!aligned16(x_q) || !aligned16(x_k)) return SCFA_EINVAL;
    if (dtype != SCFA_BF16 && dtype != SCFA_F32) return SCFA_EUNSUPPORTED;
    if (d != 64 && d != 128) return SCFA_EUNSUPPORTED;
    if (nb > SCFA_MAX_BUCKETS || (size_t)d * (nb / 2) * 4 > 64 * 1024 || S > 65535) return SCFA_EUNSUPPORTED;
    return launch_lsh_buckets(x_k ? 2 : 1, x_q, x_k, R, S, H, T, d, nb, dtype == SCFA_BF16, bucket_q_out,
                              bucket_k_out, (hipStream_t)stream);
}


int scfa_gather_rows(const void* x, const int32_t* idx, const int32_t* count, int S, int T, int d, int dtype,
                     int out_dtype, float scale, void* out, void* stream)
{
    if (!x || !idx || !out || S <= 0 || T <= 0 || d <= 0 || !isfinite(scale)) return SCFA_EINVAL;
    if (dtype != SCFA_BF16 && dtype != SCFA_F32) return SCFA_EUNSUPPORTED;
    if (out_dtype != dtype && !(dtype == SCFA_BF16 && out_dtype == SCFA_F16)) return SCFA_EUNSUPPORTED;
    if (scale != 1.0f && dtype == SCFA_BF16 && out_dtype == SCFA_BF16) return SCFA_EUNSUPPORTED;   // bf16 copies are bit-exact only
    const int mode = out_dtype != dtype ? 1 : (scale != 1.0f ? 2 : 0);
    const long long row_bytes = (long long)d * (dtype == SCFA_BF16 ? 2 : 4);
    if (row_bytes % 16 != 0 || !aligned16(x) || !aligned16(out)) return SCFA_EINVAL;
    if (S > 65535 || (long long)T * (row_bytes / 16) / 256 > 0x7fffffffLL) return SCFA_EUNSUPPORTED;
    const void* xs[1] = {x};
    const int32_t* is[1] = {idx};
    const int32_t* cs[1] = {count};
    void* os[1] = {out};
    return launch_gather_rows(1, xs, is, cs, &scale, os, S, T, (int)row_bytes, mode, (hipStream_t)stream);
}

int scfa_gather_qkv(const void* q, const void* k, const void* v, const int32_t* q_idx, const int32_t* k_idx,
                    const int32_t* n_q, const int32_t* n_k, int S, int T, int d, int dtype, int out_dtype,
                    float q_scale, void* q_out, void* k_out, void* v_out, void* stream)
{
    if (!q || !k || !v || !q_idx || !k_idx || !q_out || !k_out || !v_out || S <= 0 || T <= 0 || d <= 0 ||
        !isfinite(q_scale))
        return SCFA_EINVAL;
    if (dtype != SCFA_BF16 && dtype != SCFA_F32) return SCFA_EUNSUPPORTED;
    if (out_dtype != dtype && !(dtype == SCFA_BF16 && out_dtype == SCFA_F16)) return SCFA_EUNSUPPORTED;
    if (q_scale != 1.0f && dtype == SCFA_BF16 && out_dtype == SCFA_BF16) return SCFA_EUNSUPPORTED;
    const int mode = out_dtype != dtype ? 1 : (dtype == SCFA_F32 ? 2 : 0);
    const long long row_bytes = (long long)d * (dtype == SCFA_BF16 ? 2 : 4);
    if (row_bytes % 16 != 0 || !aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(q_out) ||
        !aligned16(k_out) || !aligned16(v_out))
        return SCFA_EINVAL;
    if (S > 65535 || (long long)T * (row_bytes / 16) / 256 > 0x7fffffffLL) return SCFA_EUNSUPPORTED;
    const void* xs[3] = {q, k, v};
    const int32_t* is[3] = {q_idx, k_idx, k_idx};
    const int32_t* cs[3] = {n_q, n_k, n_k};
    const float sc[3] = {q_scale, 1.0f, 1.0f};
    void* os[3] = {q_out, k_out, v_out};
    return launch_gather_rows(3, xs, is, cs, sc, os, S, T, (int)row_bytes, mode, (hipStream_t)stream);
}

int scfa_num_work_items(int T, int nb, int tile)
{
    if (T <= 0 || nb <= 0 || tile <= 0) return SCFA_EINVAL;
    return (T + tile - 1) / tile + nb;
}

int scfa_tile_config(int d, int dtype, int* fwd_tile_m, int* fwd_tile_n, int* bwd_tile_n, int* bwd_tile_m)
{
    if (!fwd_tile_m || !fwd_tile_n || !bwd_tile_n || !bwd_tile_m) return SCFA_EINVAL;
    if (d != 64 && d != 128) return SCFA_EUNSUPPORTED;
    if (dtype == SCFA_BF16) {
        *fwd_tile_m = FWD_TILE_M; *fwd_tile_n = FWD_TILE_N;
    } else if (dtype == SCFA_F32) {
        *fwd_tile_m = F32_TILE_M; *fwd_tile_n = F32_TILE_N;
    } else {
        return SCFA_EUNSUPPORTED;
    }
    *bwd_tile_n = BWD_TILE_N; *bwd_tile_m = BWD_TILE_M;
    return SCFA_OK;
}

int scfa_block_ranges(int variant, const int32_t* q_idx, const int32_t* k_idx, const int32_t* q_off,
                      const int32_t* k_off, int S, int T, int nb, int fwd_tile_m, int fwd_tile_n,
                      int bwd_tile_n, int bwd_tile_m, int flags, int32_t* fwd_work_out,
                      int32_t* bwd_work_out, int64_t* counters_out, void* stream)
{
    if (!q_idx || !k_idx || !q_off || !k_off || !fwd_work_out || S <= 0 || T <= 0 || nb <= 0) return SCFA_EINVAL;
    if (variant != SCFA_HASH && variant != SCFA_QKDROP) return SCFA_EINVAL;
    if (variant == SCFA_QKDROP && nb != 1) return SCFA_EINVAL;
    if ((flags & ~SCFA_FLAG_STRICT_CAUSAL) != 0) return SCFA_EUNSUPPORTED;
    if (nb > SCFA_MAX_BUCKETS) return SCFA_EUNSUPPORTED;
    const bool fwd_ok = (fwd_tile_m == FWD_TILE_M && fwd_tile_n == FWD_TILE_N) ||
                        (fwd_tile_m == F32_TILE_M && fwd_tile_n == F32_TILE_N);
    if (!fwd_ok || bwd_tile_n != BWD_TILE_N || bwd_tile_m != BWD_TILE_M) return SCFA_EUNSUPPORTED;
    const int n_fwd = scfa_num_work_items(T, nb, fwd_tile_m);
    const int n_bwd = scfa_num_work_items(T, nb, bwd_tile_n);
    if (n_fwd > 8192 || n_bwd > 8192) return SCFA_EUNSUPPORTED;   // ranking scratch lives in LDS
    return launch_block_ranges(variant, q_idx, k_idx, q_off, k_off, S, T, nb, fwd_tile_m, fwd_tile_n, bwd_tile_n,
                               bwd_tile_m, n_fwd, n_bwd, flags & SCFA_FLAG_STRICT_CAUSAL, fwd_work_out, bwd_work_out, counters_out,
                               (hipStream_t)stream);
}

int scfa_hash_attn_fwd(const void* q_perm, const void* k_perm, const void* v_perm, const uint32_t* q_sort_key,
                       const uint32_t* k_sort_key, const int32_t* fwd_work, int n_fwd, int B, int H, int T, int d,
                       int dtype, float sm_scale, int flags, void* o_out, float* lse_out, void* o_f16_out,
                       void* stream)
{
    return attn_fwd_impl(q_perm, k_perm, v_perm, q_sort_key, k_sort_key, nullptr, false, fwd_work, n_fwd, B, H, T, d, dtype,
                         sm_scale, flags, o_out, lse_out, o_f16_out, (hipStream_t)stream);
}

int scfa_qkdrop_attn_fwd(const void* q_c, const void* k_c, const void* v_c, const int32_t* q_idx,
                         const int32_t* k_idx, const int32_t* n_q, const int32_t* fwd_work, int n_fwd, int B,
                         int H, int T, int d, int dtype, float sm_scale, int flags, void* o_out, float* lse_out,
                         void* o_f16_out, void* stream)
{
    return attn_fwd_impl(q_c, k_c, v_c, reinterpret_cast<const uint32_t*>(q_idx), reinterpret_cast<const uint32_t*>(k_idx), n_q, true, fwd_work, n_fwd, B, H, T, d, dtype, sm_scale,
                         flags, o_out, lse_out, o_f16_out, (hipStream_t)stream);
}

size_t scfa_attn_bwd_workspace_bytes(int S, int T, int d, int dtype)
{
    if (S <= 0 || T <= 0 || d <= 0 || dtype != SCFA_BF16) return 0;
    return align_up((size_t)S * T * d * 2, 256) + 2 * align_up((size_t)S * T * 4, 256) +
           align_up((size_t)S * T * 16, 256) + align_up((size_t)S * 64 * 4, 256) + align_up((size_t)S * 4, 256);
}

int scfa_hash_attn_bwd(const void* q_perm, const void* k_perm, const void* v_perm, const uint32_t* q_sort_key,
                       const uint32_t* k_sort_key, const int32_t* fwd_work, int n_fwd, const int32_t* bwd_work,
                       int n_bwd, const void* o, const void* o_f16, const float* lse, const void* d_o, int B,
                       int H, int T, int d, int dtype, float sm_scale, int flags, float* dq_out, float* dk_out,
                       float* dv_out, void* ws, size_t ws_bytes, void* stream)
{
    return attn_bwd_impl(q_perm, k_perm, v_perm, q_sort_key, k_sort_key, nullptr, nullptr, false, fwd_work, n_fwd, bwd_work,
                         n_bwd, o, o_f16, lse, d_o, B, H, T, d, dtype, sm_scale, flags, dq_out, dk_out, dv_out, ws,
                         ws_bytes, (hipStream_t)stream);
}

int scfa_qkdrop_attn_bwd(const void* q_c, const void* k_c, const void* v_c, const int32_t* q_idx,
                         const int32_t* k_idx, const int32_t* n_q, const int32_t* n_k, const int32_t* fwd_work,
                         int n_fwd, const int32_t* bwd_work, int n_bwd, const void* o, const void* o_f16,
                         const float* lse, const void* d_o, int B, int H, int T, int d, int dtype, float sm_scale, int flags,
                         float* dq_out, float* dk_out, float* dv_out, void* ws, size_t ws_bytes, void* stream)
{
    return attn_bwd_impl(q_c, k_c, v_c, reinterpret_cast<const uint32_t*>(q_idx), reinterpret_cast<const uint32_t*>(k_idx), n_q, n_k, true, fwd_work, n_fwd, bwd_work, n_bwd, o, o_f16, lse, d_o,
                         B, H, T, d, dtype, sm_scale, flags, dq_out, dk_out, dv_out, ws, ws_bytes,
                         (hipStream_t)stream);
}

int scfa_prof_occupancy(int kernel_id, int d, int* workgroups_per_cu)
{
    if (!workgroups_per_cu) return SCFA_EINVAL;
    if (kernel_id == SCFA_K_FWD) return occupancy_attn_fwd_bf16(d, workgroups_per_cu);
    if (kernel_id == SCFA_K_BWD_DKDV) return occupancy_attn_bwd_dkdv_bf16(d, workgroups_per_cu);
    if (kernel_id == SCFA_K_BWD_DQ) return occupancy_attn_bwd_dq_bf16(d, workgroups_per_cu);
    return SCFA_EUNSUPPORTED;
}

int scfa_prof_enable(int on)
{
    std::lock_guard<std::mutex> lk(g_prof_mu);
    const int prev = g_prof_on ? 1 : 0;
    g_prof_on = on != 0;
    return prev;
}

int scfa_prof_reset(void)
{
    std::lock_guard<std::mutex> lk(g_prof_mu);
    for (auto& r : g_prof_recs) {
        (void)hipEventSynchronize(r.b);
        g_prof_pool.push_back(r.a);
        g_prof_pool.push_back(r.b);
    }
    g_prof_recs.clear();
    return SCFA_OK;
}

int scfa_prof_read(int kernel_id, double* total_ms, int* launches)
{
    if (!total_ms || !launches || kernel_id < 0 || kernel_id >= SCFA_K_COUNT) return SCFA_EINVAL;
    std::lock_guard<std::mutex> lk(g_prof_mu);
    double tot = 0.0;
    int n = 0;
    for (auto& r : g_prof_recs) {
        if (r.kid != kernel_id) continue;
        SCFA_HIP_TRY(hipEventSynchronize(r.b));
        float ms = 0.f;
        SCFA_HIP_TRY(hipEventElapsedTime(&ms, r.a, r.b));
        tot += ms;
        ++n;
    }
    *total_ms = tot;
    *launches = n;
    return SCFA_OK;
}

}  // extern "C"
