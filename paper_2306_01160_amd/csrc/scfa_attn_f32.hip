// fp32 forward attention over the work list: one thread per query row, keys staged
// through LDS 32 at a time, plain online softmax in fp32 (the running maximum / sum
// recurrence of paper App. B.1 with an un-normalised accumulator that is divided by
// the sum once at the end).  A key is either taken or skipped per row, so a row that
// never takes a key keeps l = 0 and writes a zero vector and LSE = -inf, which is the
// paper's treatment of stranded queries (Sec. 3.1 "Edge cases") without its
// -inf / inf replacements.  No throughput target: this is the full-precision path.
#include "scfa_common.hpp"

#include <math.h>

namespace scfa {

template <int D>
__global__ __launch_bounds__(F32_TILE_M) void attn_fwd_f32_kernel(
    const float* __restrict__ q, const float* __restrict__ k, const float* __restrict__ v,
    const uint32_t* __restrict__ q_key, const uint32_t* __restrict__ k_key,
    const int32_t* __restrict__ work, int n_work, int T, float tau, int strict, float* __restrict__ o,
    float* __restrict__ lse)
{
    __shared__ float Ks[F32_TILE_N][D];
    __shared__ float Vs[F32_TILE_N][D];
    __shared__ uint32_t kkey[F32_TILE_N];   // sort keys: bucket << 24 | position

    const int s = blockIdx.y;
    const int32_t* it = work + ((size_t)s * n_work + blockIdx.x) * WORK_STRIDE;
    const int q_begin = it[W_QBEGIN], q_count = it[W_QCOUNT];
    const int k_begin = it[W_KBEGIN], k_count = it[W_KCOUNT];
    if (q_count <= 0) return;

    const int r = threadIdx.x;
    const bool valid = r < q_count;
    const size_t seg = (size_t)s * T;
    const uint32_t qkey = valid ? q_key[seg + q_begin + r] : 0u;
    const int qpos = valid ? (int)(qkey & KEY_POS_MASK) : -1;
    // a key is taken iff (its sort key - qlo) <= qspan: same bucket, position <= the query's (< if strict)
    const bool some = valid && qpos - strict >= 0;
    const uint32_t qlo = some ? (qkey & ~KEY_POS_MASK) : KEY_NEVER;
    const uint32_t qspan = some ? (uint32_t)(qpos - strict) : 0u;

    float qr[D], acc[D];
#pragma unroll
    for (int c = 0; c < D; ++c) { qr[c] = 0.f; acc[c] = 0.f; }
    if (valid) {
        const float4* src = reinterpret_cast<const float4*>(q + (seg + q_begin + r) * D);
#pragma unroll
        for (int c = 0; c < D / 4; ++c) {
            const float4 t = src[c];
            qr[4 * c] = t.x; qr[4 * c + 1] = t.y; qr[4 * c + 2] = t.z; qr[4 * c + 3] = t.w;
        }
    }
    float m = -INFINITY, l = 0.f;

    for (int k0 = 0; k0 < k_count; k0 += F32_TILE_N) {
        __syncthreads();
        for (int e = threadIdx.x; e < F32_TILE_N * (D / 4); e += F32_TILE_M) {
            const int j = e / (D / 4), c = e % (D / 4);
            float4 kk = make_float4(0.f, 0.f, 0.f, 0.f), vv = kk;
            if (k0 + j < k_count) {
                kk = reinterpret_cast<const float4*>(k + (seg + k_begin + k0 + j) * D)[c];
                vv = reinterpret_cast<const float4*>(v + (seg + k_begin + k0 + j) * D)[c];
            }
            reinterpret_cast<float4*>(&Ks[j][0])[c] = kk;
            reinterpret_cast<float4*>(&Vs[j][0])[c] = vv;
        }
        if (threadIdx.x < F32_TILE_N)
            kkey[threadIdx.x] = (k0 + threadIdx.x < k_count) ? k_key[seg + k_begin + k0 + threadIdx.x]
                                                              : KEY_PAST_END;
        __syncthreads();
        for (int j = 0; j < F32_TILE_N; ++j) {
            if (kkey[j] - qlo > qspan) continue;   // bucket and causal test in one range test
            float sc = 0.f;
#pragma unroll
            for (int c = 0; c < D; ++c) sc = fmaf(qr[c], Ks[j][c], sc);
            sc *= tau;
            const float m_new = fmaxf(m, sc);
            const float alpha = expf(m - m_new);   // m = -inf on the first taken key -> 0
            const float p = expf(sc - m_new);
            l = l * alpha + p;
#pragma unroll
            for (int c = 0; c < D; ++c) acc[c] = fmaf(p, Vs[j][c], acc[c] * alpha);
            m = m_new;
        }
    }
    if (!valid) return;
    const float inv = l > 0.f ? 1.f / l : 0.f;
    float4* dst = reinterpret_cast<float4*>(o + (seg + qpos) * D);
#pragma unroll
    for (int c = 0; c < D / 4; ++c)
        dst[c] = make_float4(acc[4 * c] * inv, acc[4 * c + 1] * inv, acc[4 * c + 2] * inv, acc[4 * c + 3] * inv);
    lse[seg + qpos] = l > 0.f ? m + logf(l) : -INFINITY;
}

int launch_attn_fwd_f32(const float* q, const float* k, const float* v, const uint32_t* q_key,
                        const uint32_t* k_key, const int32_t* work, int n_work, int S, int T, int d,
                        float tau, int strict, float* o, float* lse, hipStream_t st)
{
    dim3 grid(n_work, S), block(F32_TILE_M);
    ProfScope prof(SCFA_K_FWD, st);
    if (d == 64)
        hipLaunchKernelGGL(attn_fwd_f32_kernel<64>, grid, block, 0, st, q, k, v, q_key, k_key, work, n_work, T, tau, strict, o, lse);
    else if (d == 128)
        hipLaunchKernelGGL(attn_fwd_f32_kernel<128>, grid, block, 0, st, q, k, v, q_key, k_key, work, n_work, T, tau, strict, o, lse);
    else
        return SCFA_EUNSUPPORTED;
    SCFA_HIP_TRY(hipGetLastError());
    return SCFA_OK;
}

}  // namespace scfa
