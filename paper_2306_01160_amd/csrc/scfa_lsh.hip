// LSH bucketing in front of the hash-sparse path (paper Sec. 4.2 "Hashing mechanism": the
// cross-polytope scheme of Andoni et al. with a chosen number of hash codes).  For every
// row x of a [S,T,d] tensor and the projection R of its head (d x r, r = nb / 2):
//     bucket = argmax over [x R, -x R]        (lowest index on ties)
// HBM-bound: x is read once (16 bytes per lane, a row is d/8 adjacent lanes), R sits in LDS,
// 4 bytes are written per row.  The r dot products are formed eight columns at a time: each
// lane multiplies its 8 elements into partial sums (its 8 x 8 block of R in registers, reused
// for eight rows), the row's lanes add them up with cross-lane shuffles, and a running
// (value, index) maximum over +-p is kept.  Arithmetic is
// fp32 (fused multiply-adds in element order inside a lane, then a pairwise tree over lanes).
#include "scfa_common.hpp"

namespace scfa {

struct LshProblem {
    const void* x;
    int32_t* bucket_out;
};

// sum over the LANES adjacent lanes of a row (8 or 16, aligned) with data-parallel-primitive moves:
// swap neighbours, swap pairs, mirror within 8 lanes, mirror within 16 lanes.  After each step the
// lanes that were combined hold the same value, so a mirror pairs complete groups.
template <int CTRL>
__device__ __forceinline__ float dpp_add(float x)
{
    const int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true);
    return x + __int_as_float(y);
}
template <int LANES>
__device__ __forceinline__ float row_sum(float x)
{
    x = dpp_add<0xB1>(x);    // quad_perm [1,0,3,2]
    x = dpp_add<0x4E>(x);    // quad_perm [2,3,0,1]
    x = dpp_add<0x141>(x);   // row_half_mirror
    if (LANES == 16) x = dpp_add<0x140>(x);   // row_mirror
    return x;
}

constexpr int LSH_ROWS = 8;   // rows per thread: the projection columns a lane needs are read from LDS once for all of them

template <int D, bool BF16>
__global__ __launch_bounds__(256) void lsh_buckets_kernel(LshProblem p0, LshProblem p1, const float* __restrict__ R,
                                                          int H, int T, int r)
{
    constexpr int LPR = D / 8;               // lanes per row
    constexpr int RPB = 256 / LPR;           // rows per workgroup and step
    extern __shared__ float s_R[];           // [D][r] of this head
    const int s = blockIdx.y;
    const LshProblem& pr = blockIdx.z ? p1 : p0;
    const float* Rh = R + (size_t)(s % H) * D * r;
    for (int i = threadIdx.x; i < D * r; i += 256) s_R[i] = Rh[i];
    __syncthreads();

    const int c8 = threadIdx.x % LPR;
    const int row0 = blockIdx.x * (RPB * LSH_ROWS) + threadIdx.x / LPR;
    float xv[LSH_ROWS][8];
#pragma unroll
    for (int u = 0; u < LSH_ROWS; ++u) {     // all loads of the thread are in flight together
        const int row = row0 + u * RPB;
        if (BF16) {
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (row < T) v = reinterpret_cast<const uint4*>(pr.x)[((size_t)s * T + row) * LPR + c8];
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                xv[u][2 * i] = __uint_as_float(w[i] << 16);
                xv[u][2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
            }
        } else {
            float4 a = make_float4(0.f, 0.f, 0.f, 0.f), b = a;
            if (row < T) {
                const float4* src = reinterpret_cast<const float4*>(pr.x) + ((size_t)s * T + row) * (D / 4) + c8 * 2;
                a = src[0]; b = src[1];
            }
            xv[u][0] = a.x; xv[u][1] = a.y; xv[u][2] = a.z; xv[u][3] = a.w;
            xv[u][4] = b.x; xv[u][5] = b.y; xv[u][6] = b.z; xv[u][7] = b.w;
        }
    }

    float best[LSH_ROWS];
    int best_idx[LSH_ROWS];
#pragma unroll
    for (int u = 0; u < LSH_ROWS; ++u) { best[u] = -INFINITY; best_idx[u] = 0; }
    for (int c0 = 0; c0 < r; c0 += 8) {
        float Rc[8][8];                       // rows 8 c8 .. 8 c8 + 7 of R, columns c0 .. c0 + 7
#pragma unroll
        for (int e = 0; e < 8; ++e)
#pragma unroll
            for (int j = 0; j < 8; ++j) Rc[e][j] = c0 + j < r ? s_R[(c8 * 8 + e) * r + c0 + j] : 0.f;
#pragma unroll
        for (int u = 0; u < LSH_ROWS; ++u) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if (c0 + j >= r) break;       // wave-uniform
                float acc = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) acc = fmaf(xv[u][e], Rc[e][j], acc);
                acc = row_sum<LPR>(acc);
                // candidates in index order: +p_c has index c, -p_c has index r + c; a strictly larger
                // value or an equal value with a lower index replaces the current choice
                const float nv = -acc;
                const int pi = c0 + j, ni = r + c0 + j;
                if (acc > best[u] || (acc == best[u] && pi < best_idx[u])) { best[u] = acc; best_idx[u] = pi; }
                if (nv > best[u] || (nv == best[u] && ni < best_idx[u])) { best[u] = nv; best_idx[u] = ni; }
            }
        }
    }
#pragma unroll
    for (int u = 0; u < LSH_ROWS; ++u) {
        const int row = row0 + u * RPB;
        if (row < T && c8 == 0) pr.bucket_out[(size_t)s * T + row] = best_idx[u];
    }
}

int launch_lsh_buckets(int n_problems, const void* x0, const void* x1, const float* R, int S, int H, int T, int d,
                       int nb, bool bf16, int32_t* out0, int32_t* out1, hipStream_t st)
{
    const int r = nb / 2;
    const size_t smem = sizeof(float) * (size_t)d * r;
    const LshProblem p0{x0, out0}, p1{x1, out1};
    const int rows_per_block = 256 / (d / 8) * LSH_ROWS;
    dim3 grid((unsigned)((T + rows_per_block - 1) / rows_per_block), S, n_problems), block(256);
    ProfScope prof(SCFA_K_LSH, st);
#define SCFA_LSH_LAUNCH(DD, BB)                                                                              \
    do {                                                                                                     \
        static std::atomic<unsigned long long> lds_allowed{0}; \
        const int rc_ = allow_dynamic_lds(reinterpret_cast<const void*>(&lsh_buckets_kernel<DD, BB>), 64 * 1024, \
                                          lds_allowed); \
        if (rc_ != SCFA_OK) return rc_; \
        hipLaunchKernelGGL((lsh_buckets_kernel<DD, BB>), grid, block, smem, st, p0, p1, R, H, T, r);         \
    } while (0)
    if (d == 64 && bf16) SCFA_LSH_LAUNCH(64, true);
    else if (d == 64) SCFA_LSH_LAUNCH(64, false);
    else if (d == 128 && bf16) SCFA_LSH_LAUNCH(128, true);
    else if (d == 128) SCFA_LSH_LAUNCH(128, false);
    else return SCFA_EUNSUPPORTED;
#undef SCFA_LSH_LAUNCH
    SCFA_HIP_TRY(hipGetLastError());
    return SCFA_OK;
}

}  // namespace scfa
