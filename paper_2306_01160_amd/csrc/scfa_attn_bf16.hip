// bf16 attention kernels for gfx950: forward, backward pre-pass, dK/dV and dQ.
//
// All three attention kernels walk a work list (scfa_block_ranges): a tile of rows
// of one bucket on the "owned" side and a contiguous range of rows of the same
// bucket on the other side.  Only the causal test on original positions is applied
// inside a tile (paper Sec. 3.1 / 3.2: "apply a causal mask locally by comparing
// indices"), and only in tiles the schedule could not prove mask-free.
//
// Matrix-core mapping (v_mfma_f32_32x32x16_bf16, 64-wide wavefronts).  A wavefront
// owns 32 rows of the owned side and keeps them in the lanes (lane % 32), so every
// per-row quantity (running max, running sum, LSE, D) is one scalar per lane and a
// row reduction is register-local plus one exchange between the lane halves:
//   forward : S^T = K_j Q_i^T  (keys x queries),  O^T += V_j^T P^T
//   dQ      : S^T, dP^T = V_j dO_i^T,  dQ^T += K_j^T dS^T
//   dK/dV   : S = Q_i K_j^T (queries x keys), dP = dO_i V_j^T,
//             dV^T += dO_i^T P,  dK^T += Q_i^T dS
// The accumulator layout of S^T (lane = column, registers = rows) is exactly the
// B-operand layout needed by the second contraction, so P / dS never leave registers.
// The other operand of the second contraction must be K-dim-major; it is staged in
// LDS transposed (pairs of rows packed in one dword, row stride 33 dwords so that
// both the transposing writes and the operand reads are bank-conflict free).
//
// Softmax (paper App. B.1, "Accumulating softmax statistics while avoiding NaNs"):
// running maximum m and running sum l per row, un-normalised accumulator rescaled by
// exp(m_old - m_new), one division at the end.  A row whose keys are all masked keeps
// m = -inf; the exponent base is then taken as 0 (the paper's replacement of -inf by 0)
// so every p is exp(-inf) = 0, l stays 0, and the row is written as zeros with
// LSE = -inf.
#include "scfa_common.hpp"

#include <math.h>

namespace scfa {

using bf16x8 = __bf16 __attribute__((ext_vector_type(8)));
using f16x8 = _Float16 __attribute__((ext_vector_type(8)));
using f16x2 = _Float16 __attribute__((ext_vector_type(2)));
using f32x16 = float __attribute__((ext_vector_type(16)));

constexpr float LOG2E = 1.4426950408889634f;

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ f16x8 as_f16x8(uint4 v) { return __builtin_bit_cast(f16x8, v); }

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ f32x16 mfma32(f16x8 a, f16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}

// two floats -> packed fp16 pair.  Round-toward-zero: never produces inf from a finite
// input (saturates at the largest fp16), relative error < 2^-10.
__device__ __forceinline__ uint32_t pack_f16(float lo, float hi)
{
    return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(lo, hi));
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ float xhalf(float x) { return __shfl_xor(x, 32); }

// registers 8*cc .. 8*cc+7 of an accumulator block as an fp16 B-operand chunk
__device__ __forceinline__ f16x8 pack_chunk(const f32x16& p, int cc)
{
    return as_f16x8(make_uint4(pack_f16(p[8 * cc + 0], p[8 * cc + 1]), pack_f16(p[8 * cc + 2], p[8 * cc + 3]),
                               pack_f16(p[8 * cc + 4], p[8 * cc + 5]), pack_f16(p[8 * cc + 6], p[8 * cc + 7])));
}

// ---------------------------------------------------------------------------
// Global -> LDS staging of a tile of ROWS rows x D bf16.  A thread owns "items":
// two adjacent rows (2p, 2p+1) x one 8-element column chunk.  The two rows can be
// stored row-major (operand with the head dimension as contraction dim) and/or
// transposed (operand with the row index as contraction dim).
template <int D, int ROWS>
struct PairTile {
    static constexpr int CHUNKS = D / 8;
    static constexpr int ITEMS = (ROWS / 2) * CHUNKS / 256;
    static_assert((ROWS / 2) * CHUNKS % 256 == 0, "tile must split evenly over 256 threads");
    uint4 lo[ITEMS], hi[ITEMS];

    __device__ __forceinline__ void load(const uint16_t* __restrict__ base, int nvalid)
    {
#pragma unroll
        for (int u = 0; u < ITEMS; ++u) {
            const int item = threadIdx.x + 256 * u;
            const int c8 = item % CHUNKS, r0 = 2 * (item / CHUNKS);
            const uint4 z = make_uint4(0u, 0u, 0u, 0u);
            lo[u] = r0 < nvalid ? *reinterpret_cast<const uint4*>(base + (size_t)r0 * D + c8 * 8) : z;
            hi[u] = r0 + 1 < nvalid ? *reinterpret_cast<const uint4*>(base + (size_t)(r0 + 1) * D + c8 * 8) : z;
        }
    }
    // row-major, row stride D+8 elements
    __device__ __forceinline__ void store_rows(uint16_t* lds) const
    {
#pragma unroll
        for (int u = 0; u < ITEMS; ++u) {
            const int item = threadIdx.x + 256 * u;
            const int c8 = item % CHUNKS, r0 = 2 * (item / CHUNKS);
            *reinterpret_cast<uint4*>(lds + r0 * (D + 8) + c8 * 8) = lo[u];
            *reinterpret_cast<uint4*>(lds + (r0 + 1) * (D + 8) + c8 * 8) = hi[u];
        }
    }
    // transposed and converted to fp16 (exact for bf16 values of normal fp16 range):
    // dword [dd * (ROWS/2+1) + p] = { x[2p][dd], x[2p+1][dd] }
    __device__ __forceinline__ void store_trans(uint32_t* lds) const
    {
        constexpr int TS = ROWS / 2 + 1;
#pragma unroll
        for (int u = 0; u < ITEMS; ++u) {
            const int item = threadIdx.x + 256 * u;
            const int c8 = item % CHUNKS, p = item / CHUNKS;
            const uint32_t a[4] = {lo[u].x, lo[u].y, lo[u].z, lo[u].w};
            const uint32_t b[4] = {hi[u].x, hi[u].y, hi[u].z, hi[u].w};
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                lds[(c8 * 8 + 2 * w) * TS + p] = pack_f16(__uint_as_float(a[w] << 16), __uint_as_float(b[w] << 16));
                lds[(c8 * 8 + 2 * w + 1) * TS + p] =
                    pack_f16(__uint_as_float(a[w] & 0xffff0000u), __uint_as_float(b[w] & 0xffff0000u));
            }
        }
    }
};

// A operand from a row-major tile: 8 consecutive elements of row `row` at column `col`
template <int D>
__device__ __forceinline__ bf16x8 lds_a_rows(const uint16_t* lds, int row, int col)
{
    return as_bf16x8(*reinterpret_cast<const uint4*>(lds + row * (D + 8) + col));
}

// A operand from a transposed tile: row dd, contraction slots { r0..r0+3, r0+8..r0+11 }
// with r0 = 16*chunk + 4*half (the slot order the accumulator layout of the first
// contraction gives to the B operand).
template <int ROWS>
__device__ __forceinline__ f16x8 lds_a_trans(const uint32_t* lds, int dd, int chunk, int half)
{
    constexpr int TS = ROWS / 2 + 1;
    const uint32_t* p = lds + dd * TS + chunk * 8 + half * 2;
    return as_f16x8(make_uint4(p[0], p[1], p[4], p[5]));
}

// ===========================================================================
// Backward pre-pass: D_i = <dO_i, O_i>, and dO, D, LSE brought into permuted order.
// One row is handled by D/8 adjacent lanes (16 bytes each).
// ===========================================================================
template <int D>
__global__ __launch_bounds__(256) void bwd_prep_bf16_kernel(
    const uint16_t* __restrict__ o, const float* __restrict__ o_f32, const float* __restrict__ lse,
    const uint16_t* __restrict__ d_o, const int32_t* __restrict__ q_idx, int T, uint16_t* __restrict__ do_perm,
    float* __restrict__ delta_perm, float* __restrict__ lse_perm)
{
    constexpr int LPR = D / 8;   // lanes per row
    const int s = blockIdx.y;
    const size_t seg = (size_t)s * T;
    const int r = (blockIdx.x * 256 + threadIdx.x) / LPR;
    const int c8 = threadIdx.x % LPR;
    const bool valid = r < T;
    float acc = 0.f;
    int src = 0;
    if (valid) {
        src = q_idx[seg + r];
        const uint4 g = *reinterpret_cast<const uint4*>(d_o + (seg + src) * D + c8 * 8);
        *reinterpret_cast<uint4*>(do_perm + (seg + r) * D + c8 * 8) = g;
        const uint32_t gw[4] = {g.x, g.y, g.z, g.w};
        float y[8];
        if (o_f32) {   // full-precision copy of O kept by the forward
            const float4 y0 = *reinterpret_cast<const float4*>(o_f32 + (seg + src) * D + c8 * 8);
            const float4 y1 = *reinterpret_cast<const float4*>(o_f32 + (seg + src) * D + c8 * 8 + 4);
            y[0] = y0.x; y[1] = y0.y; y[2] = y0.z; y[3] = y0.w; y[4] = y1.x; y[5] = y1.y; y[6] = y1.z; y[7] = y1.w;
        } else {
            const uint4 yb = *reinterpret_cast<const uint4*>(o + (seg + src) * D + c8 * 8);
            const uint32_t yw[4] = {yb.x, yb.y, yb.z, yb.w};
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                y[2 * w] = __uint_as_float(yw[w] << 16);
                y[2 * w + 1] = __uint_as_float(yw[w] & 0xffff0000u);
            }
        }
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            acc = fmaf(__uint_as_float(gw[w] << 16), y[2 * w], acc);
            acc = fmaf(__uint_as_float(gw[w] & 0xffff0000u), y[2 * w + 1], acc);
        }
    }
#pragma unroll
    for (int off = LPR / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
    if (valid && c8 == 0) {
        delta_perm[seg + r] = acc;
        lse_perm[seg + r] = lse[seg + src];
    }
}

int launch_bwd_prep_bf16(const void* o, const float* o_f32, const float* lse, const void* d_o, const int32_t* q_idx,
                         int S, int T, int d, void* do_perm, float* delta_perm, float* lse_perm,
                         hipStream_t st)
{
    const long long threads = (long long)T * (d / 8);
    dim3 grid((unsigned)((threads + 255) / 256), S), block(256);
    ProfScope prof(SCFA_K_BWD_PREP, st);
    if (d == 64)
        hipLaunchKernelGGL(bwd_prep_bf16_kernel<64>, grid, block, 0, st, (const uint16_t*)o, o_f32, lse, (const uint16_t*)d_o,
                           q_idx, T, (uint16_t*)do_perm, delta_perm, lse_perm);
    else if (d == 128)
        hipLaunchKernelGGL(bwd_prep_bf16_kernel<128>, grid, block, 0, st, (const uint16_t*)o, o_f32, lse, (const uint16_t*)d_o,
                           q_idx, T, (uint16_t*)do_perm, delta_perm, lse_perm);
    else
        return SCFA_EUNSUPPORTED;
    SCFA_HIP_TRY(hipGetLastError());
    return SCFA_OK;
}

// ===========================================================================
// dK / dV: a workgroup owns 128 keys of one bucket (32 per wavefront, in the
// lanes) and walks the query tiles that can see them.
// ===========================================================================
template <int D>
struct DkdvSmem {
    static constexpr int BM = BWD_TILE_M;
    uint16_t Qs[BM * (D + 8)];
    uint16_t Gs[BM * (D + 8)];          // dO rows
    uint32_t Qt[D * (BM / 2 + 1)];
    uint32_t Gt[D * (BM / 2 + 1)];
    float lse2[BM];                     // LSE * log2(e); +inf for rows that contribute nothing
    float delta[BM];
    int32_t qpos[BM];
};

template <int D>
__global__ __launch_bounds__(256) void attn_bwd_dkdv_bf16_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const uint16_t* __restrict__ do_perm, const float* __restrict__ lse_perm,
    const float* __restrict__ delta_perm, const int32_t* __restrict__ q_idx,
    const int32_t* __restrict__ k_idx, const int32_t* __restrict__ work, int n_work, int S, int T,
    float tau, float* __restrict__ dk, float* __restrict__ dv)
{
    constexpr int BM = BWD_TILE_M;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    DkdvSmem<D>& sm = *reinterpret_cast<DkdvSmem<D>*>(smem_raw);

    const int s = blockIdx.x % S;
    const int w = blockIdx.x / S;
    const int32_t* it = work + ((size_t)s * n_work + w) * WORK_STRIDE;
    const int k_begin = it[BW_KBEGIN], k_count = it[BW_KCOUNT];
    const int q_begin = it[BW_QBEGIN], q_count = it[BW_QCOUNT], q_masked = it[BW_QMASKED];
    if (k_count <= 0) return;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, h = lane >> 5;
    const size_t seg = (size_t)s * T;
    const int krow = wave * 32 + l32;
    const bool kvalid = krow < k_count;
    const int kpos = kvalid ? k_idx[seg + k_begin + krow] : INT32_MAX;

    bf16x8 kf[D / 16], vf[D / 16];
    {
        const uint16_t* kp = k + (seg + k_begin + krow) * D + h * 8;
        const uint16_t* vp = v + (seg + k_begin + krow) * D + h * 8;
        const uint4 z = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
        for (int kk = 0; kk < D / 16; ++kk) {
            kf[kk] = as_bf16x8(kvalid ? *reinterpret_cast<const uint4*>(kp + kk * 16) : z);
            vf[kk] = as_bf16x8(kvalid ? *reinterpret_cast<const uint4*>(vp + kk * 16) : z);
        }
    }

    f32x16 dkacc[D / 32], dvacc[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) { dkacc[db][i] = 0.f; dvacc[db][i] = 0.f; }
    const float c = tau * LOG2E;

    const uint16_t* qbase = q + (seg + q_begin) * D;
    const uint16_t* gbase = do_perm + (seg + q_begin) * D;
    const int n_tiles = (q_count + BM - 1) / BM;

    PairTile<D, BM> qt, gt;
    float lse_reg = INFINITY, delta_reg = 0.f;
    int qp_reg = -1;
    auto load_vecs = [&](int r0) {
        if (tid < BM) {
            const bool ok = r0 + tid < q_count;
            const float l = ok ? lse_perm[seg + q_begin + r0 + tid] : INFINITY;
            lse_reg = (l == -INFINITY) ? INFINITY : l * LOG2E;
            delta_reg = ok ? delta_perm[seg + q_begin + r0 + tid] : 0.f;
            qp_reg = ok ? q_idx[seg + q_begin + r0 + tid] : -1;
        }
    };
    auto store_all = [&]() {
        qt.store_rows(sm.Qs);
        qt.store_trans(sm.Qt);
        gt.store_rows(sm.Gs);
        gt.store_trans(sm.Gt);
        if (tid < BM) { sm.lse2[tid] = lse_reg; sm.delta[tid] = delta_reg; sm.qpos[tid] = qp_reg; }
    };
    if (n_tiles > 0) {
        qt.load(qbase, q_count);
        gt.load(gbase, q_count);
        load_vecs(0);
        store_all();
    }
    __syncthreads();

    for (int jt = 0; jt < n_tiles; ++jt) {
        const bool more = jt + 1 < n_tiles;
        if (more) {
            const int r0 = (jt + 1) * BM;
            qt.load(qbase + (size_t)r0 * D, q_count - r0);
            gt.load(gbase + (size_t)r0 * D, q_count - r0);
            load_vecs(r0);
        }

        // S = Q K^T and dP = dO V^T : two blocks of 32 queries x 32 keys each
        f32x16 sacc[2], pacc[2];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int i = 0; i < 16; ++i) { sacc[qb][i] = 0.f; pacc[qb][i] = 0.f; }
#pragma unroll
        for (int kk = 0; kk < D / 16; ++kk)
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                sacc[qb] = mfma32(lds_a_rows<D>(sm.Qs, qb * 32 + l32, kk * 16 + h * 8), kf[kk], sacc[qb]);
                pacc[qb] = mfma32(lds_a_rows<D>(sm.Gs, qb * 32 + l32, kk * 16 + h * 8), vf[kk], pacc[qb]);
            }

        const bool masked = jt * BM < q_masked;
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int r = qb * 32 + 8 * g + 4 * h;
                const float4 l2 = *reinterpret_cast<const float4*>(&sm.lse2[r]);
                const float4 dl = *reinterpret_cast<const float4*>(&sm.delta[r]);
                const float l2a[4] = {l2.x, l2.y, l2.z, l2.w};
                const float dla[4] = {dl.x, dl.y, dl.z, dl.w};
                int qpa[4] = {INT32_MAX, INT32_MAX, INT32_MAX, INT32_MAX};
                if (masked) {
                    const int4 qp = *reinterpret_cast<const int4*>(&sm.qpos[r]);
                    qpa[0] = qp.x; qpa[1] = qp.y; qpa[2] = qp.z; qpa[3] = qp.w;
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float p = fast_exp2(fmaf(sacc[qb][4 * g + e], c, -l2a[e]));
                    if (kpos > qpa[e]) p = 0.f;
                    sacc[qb][4 * g + e] = p;
                    pacc[qb][4 * g + e] = p * (pacc[qb][4 * g + e] - dla[e]);
                }
            }

        // dV^T += dO^T P ; dK^T += Q^T dS
#pragma unroll
        for (int c4 = 0; c4 < 4; ++c4) {
            const f16x8 pf = pack_chunk(sacc[c4 >> 1], c4 & 1);
            const f16x8 sf = pack_chunk(pacc[c4 >> 1], c4 & 1);
#pragma unroll
            for (int db = 0; db < D / 32; ++db) {
                dvacc[db] = mfma32(lds_a_trans<BM>(sm.Gt, db * 32 + l32, c4, h), pf, dvacc[db]);
                dkacc[db] = mfma32(lds_a_trans<BM>(sm.Qt, db * 32 + l32, c4, h), sf, dkacc[db]);
            }
        }

        __syncthreads();
        if (more) store_all();
        __syncthreads();
    }

    if (kvalid) {
        float* dkp = dk + (seg + kpos) * D + 4 * h;
        float* dvp = dv + (seg + kpos) * D + 4 * h;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                *reinterpret_cast<float4*>(dkp + db * 32 + 8 * g) =
                    make_float4(dkacc[db][4 * g] * tau, dkacc[db][4 * g + 1] * tau, dkacc[db][4 * g + 2] * tau, dkacc[db][4 * g + 3] * tau);
                *reinterpret_cast<float4*>(dvp + db * 32 + 8 * g) =
                    make_float4(dvacc[db][4 * g], dvacc[db][4 * g + 1], dvacc[db][4 * g + 2], dvacc[db][4 * g + 3]);
            }
    }
}

template <int D>
static int launch_dkdv_t(const void* q, const void* k, const void* v, const void* do_perm,
                         const float* lse_perm, const float* delta_perm, const int32_t* q_idx,
                         const int32_t* k_idx, const int32_t* work, int n_work, int S, int T, float tau,
                         float* dk, float* dv, hipStream_t st)
{
    const size_t smem = sizeof(DkdvSmem<D>);
    static bool attr_set = false;
    if (!attr_set) {
        SCFA_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_bwd_dkdv_bf16_kernel<D>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
        attr_set = true;
    }
    dim3 grid((unsigned)((size_t)S * n_work)), block(256);
    hipLaunchKernelGGL(attn_bwd_dkdv_bf16_kernel<D>, grid, block, smem, st, (const uint16_t*)q, (const uint16_t*)k,
                       (const uint16_t*)v, (const uint16_t*)do_perm, lse_perm, delta_perm, q_idx, k_idx, work, n_work,
                       S, T, tau, dk, dv);
    SCFA_HIP_TRY(hipGetLastError());
    return SCFA_OK;
}

int launch_attn_bwd_dkdv_bf16(const void* q, const void* k, const void* v, const void* do_perm,
                              const float* lse_perm, const float* delta_perm, const int32_t* q_idx,
                              const int32_t* k_idx, const int32_t* bwd_work, int n_bwd, int S, int T,
                              int d, float tau, float* dk, float* dv, hipStream_t st)
{
    ProfScope prof(SCFA_K_BWD_DKDV, st);
    if (d == 64)
        return launch_dkdv_t<64>(q, k, v, do_perm, lse_perm, delta_perm, q_idx, k_idx, bwd_work, n_bwd, S, T, tau, dk, dv, st);
    if (d == 128)
        return launch_dkdv_t<128>(q, k, v, do_perm, lse_perm, delta_perm, q_idx, k_idx, bwd_work, n_bwd, S, T, tau, dk, dv, st);
    return SCFA_EUNSUPPORTED;
}

// ===========================================================================
// dQ: same walk as the forward (a workgroup owns 128 queries of one bucket).
// ===========================================================================
template <int D>
struct DqSmem {
    static constexpr int BN = FWD_TILE_N;
    uint16_t Ks[BN * (D + 8)];
    uint16_t Vs[BN * (D + 8)];
    uint32_t Kt[D * (BN / 2 + 1)];
    int32_t kpos[BN];
};

template <int D>
__global__ __launch_bounds__(256) void attn_bwd_dq_bf16_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const uint16_t* __restrict__ do_perm, const float* __restrict__ lse_perm,
    const float* __restrict__ delta_perm, const int32_t* __restrict__ q_idx,
    const int32_t* __restrict__ k_idx, const int32_t* __restrict__ work, int n_work, int S, int T,
    float tau, float* __restrict__ dq)
{
    constexpr int BN = FWD_TILE_N;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    DqSmem<D>& sm = *reinterpret_cast<DqSmem<D>*>(smem_raw);

    const int s = blockIdx.x % S;
    const int w = blockIdx.x / S;
    const int32_t* it = work + ((size_t)s * n_work + w) * WORK_STRIDE;
    const int q_begin = it[W_QBEGIN], q_count = it[W_QCOUNT];
    const int k_begin = it[W_KBEGIN], k_count = it[W_KCOUNT], k_nomask = it[W_KNOMASK];
    if (q_count <= 0) return;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, h = lane >> 5;
    const size_t seg = (size_t)s * T;
    const int qrow = wave * 32 + l32;
    const bool qvalid = qrow < q_count;
    const int qpos = qvalid ? q_idx[seg + q_begin + qrow] : -1;
    float lse2 = INFINITY, delta = 0.f;
    if (qvalid) {
        const float l = lse_perm[seg + q_begin + qrow];
        lse2 = (l == -INFINITY) ? INFINITY : l * LOG2E;
        delta = delta_perm[seg + q_begin + qrow];
    }

    bf16x8 qf[D / 16], gf[D / 16];
    {
        const uint16_t* qp = q + (seg + q_begin + qrow) * D + h * 8;
        const uint16_t* gp = do_perm + (seg + q_begin + qrow) * D + h * 8;
        const uint4 z = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
        for (int kk = 0; kk < D / 16; ++kk) {
            qf[kk] = as_bf16x8(qvalid ? *reinterpret_cast<const uint4*>(qp + kk * 16) : z);
            gf[kk] = as_bf16x8(qvalid ? *reinterpret_cast<const uint4*>(gp + kk * 16) : z);
        }
    }

    f32x16 dqacc[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) dqacc[db][i] = 0.f;
    const float c = tau * LOG2E;

    const uint16_t* kbase = k + (seg + k_begin) * D;
    const uint16_t* vbase = v + (seg + k_begin) * D;
    const int32_t* kib = k_idx + seg + k_begin;
    const int n_tiles = (k_count + BN - 1) / BN;

    PairTile<D, BN> kt, vt;
    int kp_reg = INT32_MAX;
    auto store_all = [&]() {
        kt.store_rows(sm.Ks);
        kt.store_trans(sm.Kt);
        vt.store_rows(sm.Vs);
        if (tid < BN) sm.kpos[tid] = kp_reg;
    };
    if (n_tiles > 0) {
        kt.load(kbase, k_count);
        vt.load(vbase, k_count);
        if (tid < BN) kp_reg = tid < k_count ? kib[tid] : INT32_MAX;
        store_all();
    }
    __syncthreads();

    for (int jt = 0; jt < n_tiles; ++jt) {
        const bool more = jt + 1 < n_tiles;
        if (more) {
            const int r0 = (jt + 1) * BN;
            kt.load(kbase + (size_t)r0 * D, k_count - r0);
            vt.load(vbase + (size_t)r0 * D, k_count - r0);
            if (tid < BN) kp_reg = r0 + tid < k_count ? kib[r0 + tid] : INT32_MAX;
        }

        // S^T = K Q^T and dP^T = V dO^T
        f32x16 sacc[2], pacc[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) { sacc[kb][i] = 0.f; pacc[kb][i] = 0.f; }
#pragma unroll
        for (int kk = 0; kk < D / 16; ++kk)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                sacc[kb] = mfma32(lds_a_rows<D>(sm.Ks, kb * 32 + l32, kk * 16 + h * 8), qf[kk], sacc[kb]);
                pacc[kb] = mfma32(lds_a_rows<D>(sm.Vs, kb * 32 + l32, kk * 16 + h * 8), gf[kk], pacc[kb]);
            }

        const bool masked = (jt + 1) * BN > k_nomask;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                int kpa[4] = {INT32_MIN, INT32_MIN, INT32_MIN, INT32_MIN};
                if (masked) {
                    const int4 kp = *reinterpret_cast<const int4*>(&sm.kpos[kb * 32 + 8 * g + 4 * h]);
                    kpa[0] = kp.x; kpa[1] = kp.y; kpa[2] = kp.z; kpa[3] = kp.w;
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float p = fast_exp2(fmaf(sacc[kb][4 * g + e], c, -lse2));
                    if (kpa[e] > qpos) p = 0.f;
                    pacc[kb][4 * g + e] = p * (pacc[kb][4 * g + e] - delta);
                }
            }

        // dQ^T += K^T dS^T
#pragma unroll
        for (int c4 = 0; c4 < 4; ++c4) {
            const f16x8 sf = pack_chunk(pacc[c4 >> 1], c4 & 1);
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
                dqacc[db] = mfma32(lds_a_trans<BN>(sm.Kt, db * 32 + l32, c4, h), sf, dqacc[db]);
        }

        __syncthreads();
        if (more) store_all();
        __syncthreads();
    }

    if (qvalid) {
        float* dqp = dq + (seg + qpos) * D + 4 * h;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g)
                *reinterpret_cast<float4*>(dqp + db * 32 + 8 * g) =
                    make_float4(dqacc[db][4 * g] * tau, dqacc[db][4 * g + 1] * tau, dqacc[db][4 * g + 2] * tau, dqacc[db][4 * g + 3] * tau);
    }
}

template <int D>
static int launch_dq_t(const void* q, const void* k, const void* v, const void* do_perm,
                       const float* lse_perm, const float* delta_perm, const int32_t* q_idx,
                       const int32_t* k_idx, const int32_t* work, int n_work, int S, int T, float tau,
                       float* dq, hipStream_t st)
{
    const size_t smem = sizeof(DqSmem<D>);
    static bool attr_set = false;
    if (!attr_set) {
        SCFA_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_bwd_dq_bf16_kernel<D>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
        attr_set = true;
    }
    dim3 grid((unsigned)((size_t)S * n_work)), block(256);
    hipLaunchKernelGGL(attn_bwd_dq_bf16_kernel<D>, grid, block, smem, st, (const uint16_t*)q, (const uint16_t*)k,
                       (const uint16_t*)v, (const uint16_t*)do_perm, lse_perm, delta_perm, q_idx, k_idx, work, n_work,
                       S, T, tau, dq);
    SCFA_HIP_TRY(hipGetLastError());
    return SCFA_OK;
}

int launch_attn_bwd_dq_bf16(const void* q, const void* k, const void* v, const void* do_perm,
                            const float* lse_perm, const float* delta_perm, const int32_t* q_idx,
                            const int32_t* k_idx, const int32_t* fwd_work, int n_fwd, int S, int T,
                            int d, float tau, float* dq, hipStream_t st)
{
    ProfScope prof(SCFA_K_BWD_DQ, st);
    if (d == 64)
        return launch_dq_t<64>(q, k, v, do_perm, lse_perm, delta_perm, q_idx, k_idx, fwd_work, n_fwd, S, T, tau, dq, st);
    if (d == 128)
        return launch_dq_t<128>(q, k, v, do_perm, lse_perm, delta_perm, q_idx, k_idx, fwd_work, n_fwd, S, T, tau, dq, st);
    return SCFA_EUNSUPPORTED;
}

}  // namespace scfa
