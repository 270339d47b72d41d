// Backward attention over the work lists, fp16 compute format, fp32 accumulation.
//
// The paper states that the backward is obtained the same way as the forward (Sec. 3.1, 3.2):
// per block of keys, find the blocks of queries that can see it.  The gradients are those
// of masked softmax attention with P recomputed from the saved logsumexp:
//   P_ij = exp(tau s_ij - LSE_i),  dP_ij = <dO_i, V_j>,  D_i = <dO_i, O_i>,
//   dS_ij = P_ij (dP_ij - D_i),  dV_j = sum_i P_ij dO_i,  dK_j = tau sum_i dS_ij Q_i,
//   dQ_i = tau sum_j dS_ij K_j.
// Three kernels: a pre-pass (D, and dO / LSE brought into permuted order), a key-major
// kernel for dK and dV (backward work list), and a query-major kernel for dQ (forward
// work list).  Nothing is accumulated with atomics, so results are deterministic.
// As in the forward, tiles that need a mask test bucket and causality at once on the rows'
// sort keys (bucket << 24 | original position), and a wavefront skips a masked tile that
// lies entirely outside the range its own 32 rows can match.
//
// dO is multiplied by a power of two per (batch, head) segment so that its largest
// magnitude lies in [1, 2) before it is converted to fp16; the gradients are multiplied
// by the inverse power at the end.  Both scalings are exact.
//
// Queries, keys, values and dO are contracted as they are (the inputs' own values, like the forward),
// so the recomputed scores are the exact <q, k> up to fp32 accumulation and the softmax scale enters per
// element in fp32: P = 2^(tau log2(e) s - LSE log2 e).  (An earlier form folded tau log2(e) into the
// register-resident operand, rounded to fp16: one instruction per element less, but a relative 2^-12 per
// element of the scores, which at logits in the hundreds -- one outlier key row is enough -- put errors
// of 5 - 25 % into the gradients.)  The per-row subtractions of P and dS = P (dP - D) are folded into the
// contractions:
//   - where the row is a lane (dQ kernel) the exponent is one fused multiply-add with the per-lane
//     constant -LSE log2 e, and the dP accumulators start from -D;
//   - where the row is a register (dK/dV kernel) one more contraction step of 16 slots is appended:
//     the pre-pass writes, per query, LSE in raw-score units (LSE / tau) and D split into three fp16
//     pieces each (an 8-element "aux" row, see split3), and the key side of that step is the constant
//     (-2^5, -2^-5, -2^-14, 0 | 0, 0, 0, 0) for the score and (0, 0, 0, 0 | -1, -2^-11, -2^-11, 0)
//     for dP.  Products of fp16 numbers are exact in the fp32 accumulation, so the split only costs
//     the final fp32 rounding; the exponent is then one multiplication by tau log2(e).
// What is left per element is that multiplication (or fused multiply-add), one exponential, one
// product and the fp16 packing.  The dK/dV kernel needs both P and dS in fp16, so it packs P and
// dP - D and multiplies the packed pairs (v_pk_mul_f16: half an instruction per element, one more
// fp16 rounding in dS); P <= 1 keeps that product finite for any finite |dP - D| below the fp16 range.
//
// Range.  Values beyond the fp16 range arrive as infinities (the gather converts with IEEE rules), and a
// logsumexp or D beyond what the aux rows hold becomes infinite there: in all these cases the gradients
// come out non-finite rather than finite and wrong.
#include "scfa_common.hpp"
#include "scfa_mma.hpp"

#include <math.h>

#include <type_traits>

namespace scfa {

// ===========================================================================
// Pre-pass
// ===========================================================================
using f16x8h = _Float16 __attribute__((ext_vector_type(8)));
constexpr int AMAX_BLOCKS = 64;   // partial maxima per segment

// partial[s][blockIdx.x] = max |dO| over this workgroup's share of segment s, as float bits
// (non-negative floats order like unsigned integers).  No atomics, no initialisation.
__global__ __launch_bounds__(256) void dout_amax_kernel(const uint4* __restrict__ d_o, long long chunks_per_seg,
                                                        uint32_t* __restrict__ partial)
{
    const int s = blockIdx.y;
    const uint4* p = d_o + (size_t)s * chunks_per_seg;
    uint32_t m = 0;
    const long long stride = (long long)gridDim.x * 256;
    long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    for (; i + 3 * stride < chunks_per_seg; i += 4 * stride) {   // four independent loads in flight
        const uint4 v[4] = {p[i], p[i + stride], p[i + 2 * stride], p[i + 3 * stride]};
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                m = max(m, (w[j] << 16) & 0x7fffffffu);
                m = max(m, w[j] & 0x7fff0000u);
            }
        }
    }
    for (; i < chunks_per_seg; i += stride) {
        const uint4 v = p[i];
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            m = max(m, (w[j] << 16) & 0x7fffffffu);
            m = max(m, w[j] & 0x7fff0000u);
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, off));
    __shared__ uint32_t wave_max[4];
    if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0)
        partial[(size_t)s * AMAX_BLOCKS + blockIdx.x] = max(max(wave_max[0], wave_max[1]), max(wave_max[2], wave_max[3]));
}

// power-of-two scale that brings a magnitude with these float bits into [1, 2)
__device__ __forceinline__ void pow2_scales(uint32_t amax_bits, float& scale, float& inv_scale)
{
    int e = (int)((amax_bits >> 23) & 0xff);
    if (amax_bits == 0 || e == 0xff) e = 127;        // zero or non-finite: no scaling
    e = max(e, 1);
    scale = __uint_as_float((uint32_t)(254 - e) << 23);      // 2^-(e-127)
    inv_scale = __uint_as_float((uint32_t)e << 23);          // 2^(e-127)
}

// x = a1 h1 + a2 h2 + a3 h3 with fp16 h1, h2, h3 and powers of two a1 >= a2 >= a3 (all normal fp16 numbers), to
// about 33 bits; packed as (h1, h2), (h3, 0).  The residuals are exact in fp32, so a piece that rounds (or
// underflows) is made up for by the next one.  |x| beyond 65504 a1 makes h1 infinite and the gradients of that
// row non-finite: out of the kernels' range, and visibly so.  D (after the scaling of dO) uses (1, 2^-11, 2^-11):
// range 65504.  The logsumexp is stored in units of the raw scores <q, k>, LSE log2(e) / (tau log2(e)), i.e.
// about LSE / tau: (2^5, 2^-5, 2^-14) reach 2.09e6, logits of +-2.6e5 at tau = 1/8.
constexpr float AUX_D1 = 1.f, AUX_D2 = 1.f / 2048.f, AUX_D3 = 1.f / 2048.f;
constexpr float AUX_L1 = 32.f, AUX_L2 = 1.f / 32.f, AUX_L3 = 1.f / 16384.f;
constexpr float AUX_L_NO_KEYS = 2.0e6f;   // stands for LSE = -inf (a row without keys): every probability becomes 0
__device__ __forceinline__ void split3(float x, float a1, float a2, float a3, uint32_t& w01, uint32_t& w23)
{
    const _Float16 h1 = (_Float16)(x * (1.f / a1));
    const float r1 = x - (float)h1 * a1;                  // exact
    const _Float16 h2 = (_Float16)(r1 * (1.f / a2));
    const float r2 = r1 - (float)h2 * a2;                 // exact
    const _Float16 h3 = (_Float16)(r2 * (1.f / a3));
    w01 = (uint32_t)__builtin_bit_cast(uint16_t, h1) | ((uint32_t)__builtin_bit_cast(uint16_t, h2) << 16);
    w23 = (uint32_t)__builtin_bit_cast(uint16_t, h3);
}

// One row is handled by D/8 adjacent lanes (16 bytes of dO each).
template <int D>
__global__ __launch_bounds__(256) void bwd_prep_kernel(
    const uint16_t* __restrict__ o, const uint16_t* __restrict__ o_f16, const float* __restrict__ lse,
    const uint16_t* __restrict__ d_o, const uint32_t* __restrict__ q_key, const int32_t* __restrict__ n_q,
    const uint32_t* __restrict__ amax_partial,
    int n_partial, int T, float inv_cexp, uint16_t* __restrict__ do_perm, float* __restrict__ delta_perm, float* __restrict__ lse_perm,
    uint16_t* __restrict__ aux_perm, float* __restrict__ inv_scale_out)
{
    constexpr int LPR = D / 8;   // lanes per row
    const int s = blockIdx.y;
    const size_t seg = (size_t)s * T;
    const int r = (blockIdx.x * 256 + threadIdx.x) / LPR;
    const int c8 = threadIdx.x % LPR;
    const bool valid = r < (n_q ? n_q[s] : T);   // rows of dropped queries are never read by the kernels
    __shared__ uint32_t s_amax;
    if (threadIdx.x < 64) {   // reduce the segment's partial maxima
        uint32_t m = (int)threadIdx.x < n_partial ? amax_partial[(size_t)s * AMAX_BLOCKS + threadIdx.x] : 0u;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, off));
        if (threadIdx.x == 0) s_amax = m;
    }
    __syncthreads();
    float scale, inv_scale;
    pow2_scales(s_amax, scale, inv_scale);
    if (blockIdx.x == 0 && threadIdx.x == 0) inv_scale_out[s] = inv_scale;
    float acc = 0.f;
    int src = 0;
    if (valid) {
        src = (int)(q_key[seg + r] & KEY_POS_MASK);   // original position of sorted row r
        const uint4 g = *reinterpret_cast<const uint4*>(d_o + (seg + src) * D + c8 * 8);
        const uint32_t gw[4] = {g.x, g.y, g.z, g.w};
        float gs[8], y[8];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            gs[2 * w] = __uint_as_float(gw[w] << 16) * scale;
            gs[2 * w + 1] = __uint_as_float(gw[w] & 0xffff0000u) * scale;
        }
        if (o_f16) {   // fp16 copy of O kept by the forward (three more significant bits than bf16)
            const uint4 yh = *reinterpret_cast<const uint4*>(o_f16 + (seg + src) * D + c8 * 8);
            const f16x8h yv = __builtin_bit_cast(f16x8h, yh);
#pragma unroll
            for (int w = 0; w < 8; ++w) y[w] = (float)yv[w];
        } else {
            const uint4 yb = *reinterpret_cast<const uint4*>(o + (seg + src) * D + c8 * 8);
            const uint32_t yw[4] = {yb.x, yb.y, yb.z, yb.w};
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                y[2 * w] = __uint_as_float(yw[w] << 16);
                y[2 * w + 1] = __uint_as_float(yw[w] & 0xffff0000u);
            }
        }
        uint32_t out[4];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            acc = fmaf(gs[2 * w], y[2 * w], acc);
            acc = fmaf(gs[2 * w + 1], y[2 * w + 1], acc);
            const _Float16 a = (_Float16)gs[2 * w], b = (_Float16)gs[2 * w + 1];
            out[w] = (uint32_t)__builtin_bit_cast(uint16_t, a) | ((uint32_t)__builtin_bit_cast(uint16_t, b) << 16);
        }
        *reinterpret_cast<uint4*>(do_perm + (seg + r) * D + c8 * 8) = make_uint4(out[0], out[1], out[2], out[3]);
    }
#pragma unroll
    for (int off = LPR / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
    if (valid && c8 == 0) {
        const float lse_r = lse[seg + src];
        // LSE in raw-score units; a row without keys gets an offset that makes every probability 0
        const float l_raw = lse_r != -INFINITY ? fmaf(lse_r, LOG2E, -RTZ_BIAS_LOG2) * inv_cexp : AUX_L_NO_KEYS;
        // beyond what the aux pieces hold the dK/dV kernel sees infinities; the dQ kernel, which reads these
        // fp32 copies, is given an infinite D so that both report the row as out of range
        const bool out_of_range = fabsf(l_raw) > 65504.f * AUX_L1 || fabsf(acc) > 65504.f * AUX_D1;
        delta_perm[seg + r] = out_of_range ? INFINITY : acc;
        lse_perm[seg + r] = lse_r;
        uint32_t w[4];
        split3(l_raw, AUX_L1, AUX_L2, AUX_L3, w[0], w[1]);
        split3(acc, AUX_D1, AUX_D2, AUX_D3, w[2], w[3]);
        *reinterpret_cast<uint4*>(aux_perm + (seg + r) * 8) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

int launch_bwd_prep_bf16(const void* o, const void* o_f16, const float* lse, const void* d_o, const uint32_t* q_key,
                         const int32_t* n_q,
                         int S, int T, int d, float tau, void* do_perm, float* delta_perm, float* lse_perm,
                         void* aux_perm, uint32_t* amax, float* inv_scale, hipStream_t st)
{
    ProfScope prof(SCFA_K_BWD_PREP, st);
    const long long chunks = (long long)T * d / 8;
    const long long want = (chunks + 256 * 8 - 1) / (256 * 8);
    const unsigned nblk = (unsigned)(want < AMAX_BLOCKS ? want : AMAX_BLOCKS);
    hipLaunchKernelGGL(dout_amax_kernel, dim3(nblk, S), dim3(256), 0, st, (const uint4*)d_o, chunks, amax);
    const long long threads = (long long)T * (d / 8);
    dim3 grid((unsigned)((threads + 255) / 256), S), block(256);
    if (d == 64)
        hipLaunchKernelGGL(bwd_prep_kernel<64>, grid, block, 0, st, (const uint16_t*)o, (const uint16_t*)o_f16, lse, (const uint16_t*)d_o,
                           q_key, n_q, amax, (int)nblk, T, 1.f / (tau * LOG2E), (uint16_t*)do_perm, delta_perm, lse_perm, (uint16_t*)aux_perm, inv_scale);
    else if (d == 128)
        hipLaunchKernelGGL(bwd_prep_kernel<128>, grid, block, 0, st, (const uint16_t*)o, (const uint16_t*)o_f16, lse, (const uint16_t*)d_o,
                           q_key, n_q, amax, (int)nblk, T, 1.f / (tau * LOG2E), (uint16_t*)do_perm, delta_perm, lse_perm, (uint16_t*)aux_perm, inv_scale);
    else
        return SCFA_EUNSUPPORTED;
    SCFA_HIP_TRY(hipGetLastError());
    return SCFA_OK;
}

// ===========================================================================
// dK / dV: a workgroup owns 128 keys of one bucket (32 per wavefront, in the lanes)
// and walks the 64-row query tiles that can see them.  Per tile:
//   X = Q K'^T - LSE log2 e, dP' = dO V^T - D (queries x keys; lane = key, registers =
//   queries; the subtractions ride in a 16-slot contraction step on the aux rows)
//   P = 2^X, dS = P dP'
//   dV^T += dO^T P,  dK^T += Q^T dS   (d x keys; Q^T, dO^T by transposing LDS reads)
// ===========================================================================
// LDS ring of the dK/dV kernel: Q tile, dO tile, aux rows (three fp16 pieces of LSE log2 e and of D
// per query) and query positions per buffer, filled asynchronously NBUF - 1 tiles ahead
// QK-dropping: the rows of dropped tokens get zero gradients.  Entries n_keep .. T of a segment's compacted index vector
// are the dropped positions; workgroup `w` of the `n_wg` workgroups that serve the segment zeroes the fp32 rows
// n_keep + w R, + 1, ..., then n_wg R further (R = rows one pass of the workgroup covers), in up to two tensors.  Done by
// the gradient kernels themselves, after their own stores (or at once, by workgroups without work): the zeros then
// leave for memory while other workgroups compute, instead of in launches of their own in front of the kernels.
template <int D>
__device__ __forceinline__ void zero_dropped_rows(const uint32_t* __restrict__ key_seg, int n_keep, int T, int w, int n_wg,
                                                  float* __restrict__ out0, float* __restrict__ out1, size_t seg)
{
    constexpr int CPR = D / 4;            // 16-byte chunks of an fp32 row
    constexpr int R = 256 / CPR;          // rows per pass of the workgroup
    const int sub = (int)threadIdx.x / CPR, c = (int)threadIdx.x % CPR;
    const float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
    for (long long r = (long long)n_keep + (long long)w * R + sub; r < T; r += (long long)n_wg * R) {
        const size_t row = (seg + (key_seg[r] & KEY_POS_MASK)) * D;
        reinterpret_cast<float4*>(out0 + row)[c] = z;
        if (out1) reinterpret_cast<float4*>(out1 + row)[c] = z;
    }
}

template <int D>
struct DkdvRing {
    static constexpr int BM = BWD_TILE_M;
    static constexpr int TILE_ELEMS = BM * D;
    static constexpr int AUX_OFF = TILE_ELEMS * 4;            // byte offsets inside a buffer
    static constexpr int QPOS_OFF = AUX_OFF + BM * 16;
    static constexpr int BUF_BYTES = QPOS_OFF + BM * 4;
    static constexpr int NBUF = D == 64 ? 3 : 2;
};

template <int D>
__global__ __launch_bounds__(256) void attn_bwd_dkdv_f16_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const uint16_t* __restrict__ do_perm, const uint16_t* __restrict__ aux_perm,
    const float* __restrict__ inv_scale,
    const uint32_t* __restrict__ q_key, const uint32_t* __restrict__ k_key,
    const int32_t* __restrict__ work, int n_work, int S, int T, float tau, int strict,
    float* __restrict__ dk, float* __restrict__ dv, const int32_t* __restrict__ n_keep_k)
{
    constexpr int BM = BWD_TILE_M;
    extern __shared__ __attribute__((aligned(256))) unsigned char smem_raw[];   // the hand-ordered d = 128 tile XORs address bits below 256
    using Ring = DkdvRing<D>;
    constexpr int NBUF = Ring::NBUF, BUF_BYTES = Ring::BUF_BYTES;
    constexpr int RPW = BM / 4;                                               // aux rows / positions loaded per wavefront
    constexpr int LOADS_PER_TILE = 2 * AsyncTile<D, BM, 256>::ROUNDS + 2;     // per wavefront
    auto q_tile = [&](int buf) { return reinterpret_cast<const uint16_t*>(smem_raw + buf * BUF_BYTES); };
    auto g_tile = [&](int buf) { return reinterpret_cast<const uint16_t*>(smem_raw + buf * BUF_BYTES + Ring::TILE_ELEMS * 2); };
    auto aux_tile = [&](int buf) { return reinterpret_cast<const uint16_t*>(smem_raw + buf * BUF_BYTES + Ring::AUX_OFF); };
    auto qpos_tile = [&](int buf) { return reinterpret_cast<const uint32_t*>(smem_raw + buf * BUF_BYTES + Ring::QPOS_OFF); };
    const uint32_t lds0 = lds_address(smem_raw);

    const int s = blockIdx.x % S;
    const int w = blockIdx.x / S;
    const int32_t* it = work + ((size_t)s * n_work + w) * WORK_STRIDE;
    const int k_begin = it[BW_KBEGIN], k_count = it[BW_KCOUNT];
    const int q_begin = it[BW_QBEGIN], q_count = it[BW_QCOUNT], q_masked = it[BW_QMASKED];
    if (k_count <= 0) {   // no work: only the share of the dropped rows (n_keep_k: QK-dropping, else null)
        if (n_keep_k) zero_dropped_rows<D>(k_key + (size_t)s * T, n_keep_k[s], T, w, n_work, dk, dv, (size_t)s * T);
        return;
    }

    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, l32 = lane & 31, h = lane >> 5;
    const size_t seg = (size_t)s * T;
    if (n_keep_k) zero_dropped_rows<D>(k_key + seg, n_keep_k[s], T, w, n_work, dk, dv, seg);
    const float cexp = tau * LOG2E;   // scores are raw <q, k> sums minus LSE in the same units: P = 2^(cexp x)
    const int krow = wave * 32 + l32;
    const bool kvalid = krow < k_count;
    const int kr = min(krow, k_count - 1);            // keys past the end repeat the last one; never written
    const uint32_t kkey = k_key[seg + k_begin + kr];
    const int kpos = (int)(kkey & KEY_POS_MASK);
    // a query is allowed iff (its sort key - klo) <= kspan: same bucket, position >= the key's (> if strict)
    const uint32_t klo = kvalid ? kkey + (uint32_t)strict : KEY_NEVER;
    const uint32_t kspan = kvalid ? KEY_POS_MASK - (uint32_t)(kpos + strict) : 0u;

    f16x8 kf[D / 16], vf[D / 16];
    {
        const uint16_t* kp = k + (seg + k_begin + kr) * D + h * 8;
        const uint16_t* vp = v + (seg + k_begin + kr) * D + h * 8;
#pragma unroll
        for (int kk = 0; kk < D / 16; ++kk) {
            kf[kk] = as_f16x8(*reinterpret_cast<const uint4*>(kp + kk * 16));
            vf[kk] = as_f16x8(*reinterpret_cast<const uint4*>(vp + kk * 16));
        }
#pragma unroll
        for (int kk = 0; kk < D / 16; ++kk) { touch(kf[kk]); touch(vf[kk]); }
    }

    // key side of the appended contraction step (lanes 32-63 hold slots 8-15: all zero)
    f16x8 sub_lse, sub_delta;
    {
        const _Float16 z = (_Float16)0.f;
        const _Float16 l1 = h == 0 ? (_Float16)-AUX_L1 : z, l2 = h == 0 ? (_Float16)-AUX_L2 : z, l3 = h == 0 ? (_Float16)-AUX_L3 : z;
        const _Float16 d1 = h == 0 ? (_Float16)-AUX_D1 : z, d2 = h == 0 ? (_Float16)-AUX_D2 : z, d3 = h == 0 ? (_Float16)-AUX_D3 : z;
        sub_lse = f16x8{l1, l2, l3, z, z, z, z, z};
        sub_delta = f16x8{z, z, z, z, d1, d2, d3, z};
        touch(sub_lse); touch(sub_delta);
    }

    f32x16 dkacc[D / 32], dvacc[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db) { dkacc[db] = zero16(); dvacc[db] = zero16(); }

    const int n_tiles = (q_count + BM - 1) / BM;
    const int n_masked = min((q_masked + BM - 1) / BM, n_tiles);   // leading tiles that need the causal test
    // the sort keys of the queries that may see any key of this wavefront lie in [klo_wave, khi_wave]
    uint32_t klo_wave = kvalid ? klo : 0xffffffffu, khi_wave = kvalid ? (kkey | KEY_POS_MASK) : 0u;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        klo_wave = min(klo_wave, (uint32_t)__shfl_xor((int)klo_wave, off));
        khi_wave = max(khi_wave, (uint32_t)__shfl_xor((int)khi_wave, off));
    }
    klo_wave = __builtin_amdgcn_readfirstlane(klo_wave);
    khi_wave = __builtin_amdgcn_readfirstlane(khi_wave);

    AsyncTile<D, BM, 256> loader;
    loader.init();
    const u32x4 q_desc = make_desc(q + (seg + q_begin) * D, (uint32_t)q_count * D * 2);
    const u32x4 g_desc = make_desc(do_perm + (seg + q_begin) * D, (uint32_t)q_count * D * 2);
    const u32x4 a_desc = make_desc(aux_perm + (seg + q_begin) * 8, (uint32_t)q_count * 16);
    const u32x4 p_desc = make_desc(q_key + seg + q_begin, (uint32_t)q_count * 4);
    // Every wavefront issues the same number of loads per tile, so one vmcnt threshold serves all.
    // Rows past the end of the range (and whole tiles past the end) land as zeros everywhere (Q, dO,
    // aux, positions): P = 1 there, but dO = 0 and dP' = 0 make their contributions to dV and dK
    // vanish, with or without the causal test.
    auto issue = [&](int jt, int buf) {
        const uint32_t base = lds0 + (uint32_t)(buf * BUF_BYTES);
        loader.load(q_desc, jt * loader.TILE_BYTES, base);
        loader.load(g_desc, jt * loader.TILE_BYTES, base + Ring::TILE_ELEMS * 2);
        if (lane < RPW) {
            async_load16(a_desc, __builtin_amdgcn_readfirstlane(base + Ring::AUX_OFF + wave * RPW * 16),
                         (wave * RPW + lane) * 16, jt * BM * 16);
            async_load4(p_desc, __builtin_amdgcn_readfirstlane(base + Ring::QPOS_OFF + wave * RPW * 4),
                        (wave * RPW + lane) * 4, jt * BM * 4);
        }
    };

    // The same loads one at a time (Q rounds, dO rounds, aux rows, positions), for the hand-ordered tile below, which
    // issues them between its groups: the address unit takes 16 cycles per 64-lane load, the four wavefronts of a
    // workgroup that all issue a tile's ten loads right after the barrier queue up behind each other, and with one
    // wavefront per SIMD nobody computes meanwhile.
    constexpr int ROUNDS = AsyncTile<D, BM, 256>::ROUNDS;
    auto issue_part = [&](int jt, int buf, int part) __attribute__((always_inline)) {
        const uint32_t base = lds0 + (uint32_t)(buf * BUF_BYTES);
        if (part < ROUNDS) loader.load_round(q_desc, jt * loader.TILE_BYTES, base, part);
        else if (part < 2 * ROUNDS) loader.load_round(g_desc, jt * loader.TILE_BYTES, base + Ring::TILE_ELEMS * 2, part - ROUNDS);
        else if (lane < RPW) {
            if (part == 2 * ROUNDS)
                async_load16(a_desc, __builtin_amdgcn_readfirstlane(base + Ring::AUX_OFF + wave * RPW * 16),
                             (wave * RPW + lane) * 16, jt * BM * 16);
            else
                async_load4(p_desc, __builtin_amdgcn_readfirstlane(base + Ring::QPOS_OFF + wave * RPW * 4),
                            (wave * RPW + lane) * 4, jt * BM * 4);
        }
    };

    // ---- d = 128, mask-free tiles: the vector work in the shadow of the matrix instructions --------------------
    // One wavefront per SIMD: nobody else fills the matrix core while this wavefront runs its exponentials, so the tile is
    // ordered by hand.  The scores of the first 32 queries are formed as usual; their exponentials, packing and dS then run
    // between the matrix instructions that form the scores of the other 32 queries, and the vector work of those runs between
    // the dV / dK products of the first 32.  A group = four matrix instructions (six in the first, which starts the accumulators
    // with the aux step) and the 14 vector instructions of four score elements, three or four of them after each matrix
    // instruction; the compiler's scheduler puts the phases one after the other, so the groups are inline assembly on registers
    // named in the text (scores S0 / P0 / S1 / P1 at v192-v255, packed P and dS of the four 16-query chunks at v160-v191).
    // The text knows nothing about hazards: dependent matrix instructions are two apart, a group whose vector instructions read
    // scores that matrix instructions have just written starts with a wait, an exponential is read three or more instructions later.
#define SCFA_DK_HALF(X0, X1, X2, X3, D0, D1, D2, D3, W0, W1, E0, E1, M0, M1, M2, M3, L0, L1)                                           \
    M0 L0 "v_mul_f32 " X0 ", %[c], " X0 "\n\t v_mul_f32 " X1 ", %[c], " X1 "\n\t v_mul_f32 " X2 ", %[c], " X2 "\n\t"                    \
    M1 L1 "v_mul_f32 " X3 ", %[c], " X3 "\n\t v_exp_f32 " X0 ", " X0 "\n\t v_exp_f32 " X1 ", " X1 "\n\t v_exp_f32 " X2 ", " X2 "\n\t"     \
    M2 "v_exp_f32 " X3 ", " X3 "\n\t v_cvt_pkrtz_f16_f32 " D0 ", " D0 ", " D1 "\n\t v_cvt_pkrtz_f16_f32 " D2 ", " D2 ", " D3 "\n\t"          \
    M3 "v_cvt_pkrtz_f16_f32 " W0 ", " X0 ", " X1 "\n\t v_cvt_pkrtz_f16_f32 " W1 ", " X2 ", " X3 "\n\t"                                   \
    "v_pk_mul_f16 " E0 ", " W0 ", " D0 "\n\t v_pk_mul_f16 " E1 ", " W1 ", " D2 "\n\t s_waitcnt lgkmcnt(0)\n\t"
    // The LDS reads of the NEXT group's fragments ride in the text too (L0 after the first, L1 after the second matrix instruction;
    // the group ends with their wait, which they have met by then): issued by the compiler between the groups they were a burst of
    // four to eight reads during which no matrix instruction could be issued.  Fragment sets fa / fb live at v128-v143 / v144-v159.
    // Rows of Q and dO (other 32 queries) for two steps of the head dimension: %[ra] addresses the even step, ^ 32 bytes the odd one;
    // dO tiles lie 16384 bytes behind Q tiles.
#define SCFA_DK_L_ROWS(F0, F1, F2, F3)                                                                                                  \
    "ds_read_b128 " F0 ", %[ra]\n\t ds_read_b128 " F1 ", %[ra] offset:16384\n\t",                                                     \
    "v_xor_b32 %[t0], 32, %[ra]\n\t ds_read_b128 " F2 ", %[t0]\n\t ds_read_b128 " F3 ", %[t0] offset:16384\n\t"
    // Transposed dO and Q fragments of one 16-query chunk (byte offsets OG, OQ of the chunk in the dO and Q tiles) for two 32-wide blocks
    // of the head dimension: %[ta], %[tb] address the two reads of the even block, ^ 64 bytes those of the odd one.
#define SCFA_DK_L_TRANS(F0L, F0H, F1L, F1H, F2L, F2H, F3L, F3H, OG, OQ)                                                                  \
    "ds_read_b64_tr_b16 " F0L ", %[ta] offset:" OG "\n\t ds_read_b64_tr_b16 " F0H ", %[tb] offset:" OG "\n\t"                          \
    "ds_read_b64_tr_b16 " F1L ", %[ta] offset:" OQ "\n\t ds_read_b64_tr_b16 " F1H ", %[tb] offset:" OQ "\n\t",                         \
    "v_xor_b32 %[t0], 64, %[ta]\n\t v_xor_b32 %[t1], 64, %[tb]\n\t"                                                                  \
    "ds_read_b64_tr_b16 " F2L ", %[t0] offset:" OG "\n\t ds_read_b64_tr_b16 " F2H ", %[t1] offset:" OG "\n\t"                          \
    "ds_read_b64_tr_b16 " F3L ", %[t0] offset:" OQ "\n\t ds_read_b64_tr_b16 " F3H ", %[t1] offset:" OQ "\n\t"
#define SCFA_DK_L_ROWS_(...) SCFA_DK_L_ROWS(__VA_ARGS__)
#define SCFA_DK_L_TRANS_(...) SCFA_DK_L_TRANS(__VA_ARGS__)
#define SCFA_FA_ROWS "v[128:131]", "v[132:135]", "v[136:139]", "v[140:143]"
#define SCFA_FB_ROWS "v[144:147]", "v[148:151]", "v[152:155]", "v[156:159]"
#define SCFA_FA_PAIRS "v[128:129]", "v[130:131]", "v[132:133]", "v[134:135]", "v[136:137]", "v[138:139]", "v[140:141]", "v[142:143]"
#define SCFA_FB_PAIRS "v[144:145]", "v[146:147]", "v[148:149]", "v[150:151]", "v[152:153]", "v[154:155]", "v[156:157]", "v[158:159]"
#define SCFA_FA_OUT "=&{v[128:131]}"(fa[0]), "=&{v[132:135]}"(fa[1]), "=&{v[136:139]}"(fa[2]), "=&{v[140:143]}"(fa[3])
#define SCFA_FB_OUT "=&{v[144:147]}"(fb[0]), "=&{v[148:151]}"(fb[1]), "=&{v[152:155]}"(fb[2]), "=&{v[156:159]}"(fb[3])
#define SCFA_DK_R_S0 "{v[192:207]}"
#define SCFA_DK_R_P0 "{v[208:223]}"
#define SCFA_DK_R_S1 "{v[224:239]}"
#define SCFA_DK_R_P1 "{v[240:255]}"
#define SCFA_DK_R_PF(c) "{v[" #c "]}"
    // scores of the second 32 queries, two steps of the head dimension: S1 += Qrow K, P1 += dOrow V
#define SCFA_DK_M_S                                                                                                                  \
    "v_mfma_f32_32x32x16_f16 v[224:239], %[f0], %[k0], v[224:239]\n\t", "v_mfma_f32_32x32x16_f16 v[240:255], %[f1], %[v0], v[240:255]\n\t", \
    "v_mfma_f32_32x32x16_f16 v[224:239], %[f2], %[k1], v[224:239]\n\t", "v_mfma_f32_32x32x16_f16 v[240:255], %[f3], %[v1], v[240:255]\n\t"
    // dV^T += dO^T P, dK^T += Q^T dS for one 16-query chunk and two 32-wide blocks of the head dimension
#define SCFA_DK_M_G                                                                                                                  \
    "v_mfma_f32_32x32x16_f16 %[a0], %[f0], %[pf], %[a0]\n\t", "v_mfma_f32_32x32x16_f16 %[a1], %[f1], %[sf], %[a1]\n\t",                 \
    "v_mfma_f32_32x32x16_f16 %[a2], %[f2], %[pf], %[a2]\n\t", "v_mfma_f32_32x32x16_f16 %[a3], %[f3], %[sf], %[a3]\n\t"
#define SCFA_DK_HALF_(...) SCFA_DK_HALF(__VA_ARGS__)
    const float cexp_u = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, cexp)));
    auto pin = [&]() __attribute__((always_inline)) { asm volatile("" ::: "memory"); };   // LDS reads stay on their side
    auto tile_d128 = [&](int buf, auto, int jt_next, int buf_next) __attribute__((always_inline)) {   // generic: only instantiated at d = 128
        const uint16_t* Qt = q_tile(buf);
        const uint16_t* Gt = g_tile(buf);
        const uint16_t* At = aux_tile(buf);
        f32x16 S0, P0, S1, P1;
        f16x8 pf0, sf0, pf1, sf1, pf2, sf2, pf3, sf3;
        // rows of Q and dO for two steps of the head dimension (Q, dO, Q, dO)
        auto rows2 = [&](f16x8 (&f)[4], int qb, int kk0) __attribute__((always_inline)) {
            f[0] = swz_rows<D>(Qt, qb * 32 + l32, kk0 * 16 + h * 8);
            f[1] = swz_rows<D>(Gt, qb * 32 + l32, kk0 * 16 + h * 8);
            f[2] = swz_rows<D>(Qt, qb * 32 + l32, (kk0 + 1) * 16 + h * 8);
            f[3] = swz_rows<D>(Gt, qb * 32 + l32, (kk0 + 1) * 16 + h * 8);
        };
        f16x8 fa[4], fb[4], ax1;
        // first 32 queries: aux step, then the head dimension with the row fragments one step ahead
        {
            const f16x8 ax = as_f16x8(*reinterpret_cast<const uint4*>(&At[l32 * 8]));
            S0 = mfma16(ax, sub_lse, zero16());
            P0 = mfma16(ax, sub_delta, zero16());
            rows2(fa, 0, 0);
            // one LDS read (and every other time one asynchronous load) after each matrix instruction: a burst of four
            // reads and two loads between groups of four matrix instructions lets the matrix core run dry.  The last group
            // requests the first rows of the other 32 queries before its matrix instructions: the next stage starts with them.
#pragma unroll
            for (int g = 0; g < D / 32; ++g) {
                const f16x8 (&f)[4] = (g & 1) ? fb : fa;
                f16x8 (&n)[4] = (g & 1) ? fa : fb;
                const bool last = g + 1 == D / 32;
                const int nqb = last ? 1 : 0, nkk = last ? 0 : 2 * g + 2;
                __builtin_amdgcn_sched_barrier(0);
                if (last) {
                    n[0] = swz_rows<D>(Qt, nqb * 32 + l32, nkk * 16 + h * 8);
                    n[1] = swz_rows<D>(Gt, nqb * 32 + l32, nkk * 16 + h * 8);
                    n[2] = swz_rows<D>(Qt, nqb * 32 + l32, (nkk + 1) * 16 + h * 8);
                    n[3] = swz_rows<D>(Gt, nqb * 32 + l32, (nkk + 1) * 16 + h * 8);
                    ax1 = as_f16x8(*reinterpret_cast<const uint4*>(&At[(32 + l32) * 8]));
                    __builtin_amdgcn_sched_barrier(0);
                }
                S0 = mfma16(f[0], kf[2 * g], S0);
                __builtin_amdgcn_sched_barrier(0);
                if (!last) n[0] = swz_rows<D>(Qt, nqb * 32 + l32, nkk * 16 + h * 8);
                issue_part(jt_next, buf_next, 2 * g);        // two of the eight Q and dO rounds per step
                __builtin_amdgcn_sched_barrier(0);
                P0 = mfma16(f[1], vf[2 * g], P0);
                __builtin_amdgcn_sched_barrier(0);
                if (!last) n[1] = swz_rows<D>(Gt, nqb * 32 + l32, nkk * 16 + h * 8);
                __builtin_amdgcn_sched_barrier(0);
                S0 = mfma16(f[2], kf[2 * g + 1], S0);
                __builtin_amdgcn_sched_barrier(0);
                if (!last) n[2] = swz_rows<D>(Qt, nqb * 32 + l32, (nkk + 1) * 16 + h * 8);
                issue_part(jt_next, buf_next, 2 * g + 1);
                __builtin_amdgcn_sched_barrier(0);
                P0 = mfma16(f[3], vf[2 * g + 1], P0);
                __builtin_amdgcn_sched_barrier(0);
                if (!last) n[3] = swz_rows<D>(Gt, nqb * 32 + l32, (nkk + 1) * 16 + h * 8);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // fa = rows of the other 32 queries, steps 0 and 1
        // byte addresses inside LDS (the tile ring is 256-byte aligned, so head-dimension steps and blocks are XORs of address bits)
        static_assert(D != 128 || (Ring::TILE_ELEMS * 2 == 16384 && BUF_BYTES % 256 == 0), "offsets written into the assembly text");
        const uint32_t rb = lds_address(Qt) + 2u * (uint32_t)swz_offset<D>(32 + l32, h * 8);
        int oa0, ob0;
        swz_trans_offsets<D>(0, 0, lane, oa0, ob0);
        const uint32_t ta = lds_address(Qt) + 2u * (uint32_t)oa0, tb = lds_address(Qt) + 2u * (uint32_t)ob0;
        uint32_t t0, t1;
        asm volatile("v_mfma_f32_32x32x16_f16 v[224:239], %[ax], %[sl], 0\n\t v_mfma_f32_32x32x16_f16 v[240:255], %[ax], %[sd], 0\n\t s_nop 7\n\t"
                     SCFA_DK_HALF_("v192", "v193", "v194", "v195", "v208", "v209", "v210", "v211", "v160", "v161", "v164", "v165", SCFA_DK_M_S, SCFA_DK_L_ROWS_(SCFA_FB_ROWS))
                     : "+" SCFA_DK_R_S0(S0), "+" SCFA_DK_R_P0(P0), "=&" SCFA_DK_R_S1(S1), "=&" SCFA_DK_R_P1(P1), "=&{v[160:163]}"(pf0), "=&{v[164:167]}"(sf0),
                       SCFA_FB_OUT, [t0] "=&v"(t0)
                     : [c] "s"(cexp_u), [ax] "v"(ax1), [sl] "v"(sub_lse), [sd] "v"(sub_delta), [f0] "v"(fa[0]), [f1] "v"(fa[1]), [f2] "v"(fa[2]), [f3] "v"(fa[3]),
                       [k0] "v"(kf[0]), [v0] "v"(vf[0]), [k1] "v"(kf[1]), [v1] "v"(vf[1]), [ra] "v"(rb ^ 64u));
        pin(); issue_part(jt_next, buf_next, 8); pin();
        asm volatile(SCFA_DK_HALF_("v196", "v197", "v198", "v199", "v212", "v213", "v214", "v215", "v162", "v163", "v166", "v167", SCFA_DK_M_S, SCFA_DK_L_ROWS_(SCFA_FA_ROWS))
                     : "+" SCFA_DK_R_S0(S0), "+" SCFA_DK_R_P0(P0), "+" SCFA_DK_R_S1(S1), "+" SCFA_DK_R_P1(P1), "+{v[160:163]}"(pf0), "+{v[164:167]}"(sf0),
                       SCFA_FA_OUT, [t0] "=&v"(t0)
                     : [c] "s"(cexp_u), [f0] "v"(fb[0]), [f1] "v"(fb[1]), [f2] "v"(fb[2]), [f3] "v"(fb[3]),
                       [k0] "v"(kf[2]), [v0] "v"(vf[2]), [k1] "v"(kf[3]), [v1] "v"(vf[3]), [ra] "v"(rb ^ 128u));
        pin(); issue_part(jt_next, buf_next, 9); pin();
        asm volatile(SCFA_DK_HALF_("v200", "v201", "v202", "v203", "v216", "v217", "v218", "v219", "v168", "v169", "v172", "v173", SCFA_DK_M_S, SCFA_DK_L_ROWS_(SCFA_FB_ROWS))
                     : "+" SCFA_DK_R_S0(S0), "+" SCFA_DK_R_P0(P0), "+" SCFA_DK_R_S1(S1), "+" SCFA_DK_R_P1(P1), "=&{v[168:171]}"(pf1), "=&{v[172:175]}"(sf1),
                       SCFA_FB_OUT, [t0] "=&v"(t0)
                     : [c] "s"(cexp_u), [f0] "v"(fa[0]), [f1] "v"(fa[1]), [f2] "v"(fa[2]), [f3] "v"(fa[3]),
                       [k0] "v"(kf[4]), [v0] "v"(vf[4]), [k1] "v"(kf[5]), [v1] "v"(vf[5]), [ra] "v"(rb ^ 192u));
        asm volatile(SCFA_DK_HALF_("v204", "v205", "v206", "v207", "v220", "v221", "v222", "v223", "v170", "v171", "v174", "v175", SCFA_DK_M_S,
                                   SCFA_DK_L_TRANS_(SCFA_FA_PAIRS, "16384", "0"))
                     : "+" SCFA_DK_R_S0(S0), "+" SCFA_DK_R_P0(P0), "+" SCFA_DK_R_S1(S1), "+" SCFA_DK_R_P1(P1), "+{v[168:171]}"(pf1), "+{v[172:175]}"(sf1),
                       SCFA_FA_OUT, [t0] "=&v"(t0), [t1] "=&v"(t1)
                     : [c] "s"(cexp_u), [f0] "v"(fb[0]), [f1] "v"(fb[1]), [f2] "v"(fb[2]), [f3] "v"(fb[3]),
                       [k0] "v"(kf[6]), [v0] "v"(vf[6]), [k1] "v"(kf[7]), [v1] "v"(vf[7]), [ta] "v"(ta), [tb] "v"(tb));
        // the other 32 queries' vector work under the dV / dK products of the first 16-query chunks
        asm volatile("s_nop 7\n\t"
                     SCFA_DK_HALF_("v224", "v225", "v226", "v227", "v240", "v241", "v242", "v243", "v176", "v177", "v180", "v181", SCFA_DK_M_G,
                                   SCFA_DK_L_TRANS_(SCFA_FB_PAIRS, "16384", "0"))
                     : "+" SCFA_DK_R_S1(S1), "+" SCFA_DK_R_P1(P1), "=&{v[176:179]}"(pf2), "=&{v[180:183]}"(sf2),
                       [a0] "+a"(dvacc[0]), [a1] "+a"(dkacc[0]), [a2] "+a"(dvacc[1]), [a3] "+a"(dkacc[1]), SCFA_FB_OUT, [t0] "=&v"(t0), [t1] "=&v"(t1)
                     : [c] "s"(cexp_u), [f0] "v"(fa[0]), [f1] "v"(fa[1]), [f2] "v"(fa[2]), [f3] "v"(fa[3]), [pf] "{v[160:163]}"(pf0), [sf] "{v[164:167]}"(sf0),
                       [ta] "v"(ta ^ 128u), [tb] "v"(tb ^ 128u));
        asm volatile(SCFA_DK_HALF_("v228", "v229", "v230", "v231", "v244", "v245", "v246", "v247", "v178", "v179", "v182", "v183", SCFA_DK_M_G,
                                   SCFA_DK_L_TRANS_(SCFA_FA_PAIRS, "20480", "4096"))
                     : "+" SCFA_DK_R_S1(S1), "+" SCFA_DK_R_P1(P1), "+{v[176:179]}"(pf2), "+{v[180:183]}"(sf2),
                       [a0] "+a"(dvacc[2]), [a1] "+a"(dkacc[2]), [a2] "+a"(dvacc[3]), [a3] "+a"(dkacc[3]), SCFA_FA_OUT, [t0] "=&v"(t0), [t1] "=&v"(t1)
                     : [c] "s"(cexp_u), [f0] "v"(fb[0]), [f1] "v"(fb[1]), [f2] "v"(fb[2]), [f3] "v"(fb[3]), [pf] "{v[160:163]}"(pf0), [sf] "{v[164:167]}"(sf0),
                       [ta] "v"(ta), [tb] "v"(tb));
        asm volatile(SCFA_DK_HALF_("v232", "v233", "v234", "v235", "v248", "v249", "v250", "v251", "v184", "v185", "v188", "v189", SCFA_DK_M_G,
                                   SCFA_DK_L_TRANS_(SCFA_FB_PAIRS, "20480", "4096"))
                     : "+" SCFA_DK_R_S1(S1), "+" SCFA_DK_R_P1(P1), "=&{v[184:187]}"(pf3), "=&{v[188:191]}"(sf3),
                       [a0] "+a"(dvacc[0]), [a1] "+a"(dkacc[0]), [a2] "+a"(dvacc[1]), [a3] "+a"(dkacc[1]), SCFA_FB_OUT, [t0] "=&v"(t0), [t1] "=&v"(t1)
                     : [c] "s"(cexp_u), [f0] "v"(fa[0]), [f1] "v"(fa[1]), [f2] "v"(fa[2]), [f3] "v"(fa[3]), [pf] "{v[168:171]}"(pf1), [sf] "{v[172:175]}"(sf1),
                       [ta] "v"(ta ^ 128u), [tb] "v"(tb ^ 128u));
        asm volatile(SCFA_DK_HALF_("v236", "v237", "v238", "v239", "v252", "v253", "v254", "v255", "v186", "v187", "v190", "v191", SCFA_DK_M_G,
                                   SCFA_DK_L_TRANS_(SCFA_FA_PAIRS, "24576", "8192"))
                     : "+" SCFA_DK_R_S1(S1), "+" SCFA_DK_R_P1(P1), "+{v[184:187]}"(pf3), "+{v[188:191]}"(sf3),
                       [a0] "+a"(dvacc[2]), [a1] "+a"(dkacc[2]), [a2] "+a"(dvacc[3]), [a3] "+a"(dkacc[3]), SCFA_FA_OUT, [t0] "=&v"(t0), [t1] "=&v"(t1)
                     : [c] "s"(cexp_u), [f0] "v"(fb[0]), [f1] "v"(fb[1]), [f2] "v"(fb[2]), [f3] "v"(fb[3]), [pf] "{v[168:171]}"(pf1), [sf] "{v[172:175]}"(sf1),
                       [ta] "v"(ta), [tb] "v"(tb));
        // dV / dK products of the last two 16-query chunks, fragments one step ahead
#pragma unroll
        for (int g = 0; g < 4; ++g) {       // (chunk 2, blocks 0-1), (chunk 2, blocks 2-3), (chunk 3, 0-1), (chunk 3, 2-3)
            const int c4 = 2 + (g >> 1), db0 = 2 * (g & 1);
            const int nc4 = 2 + ((g + 1) >> 1), ndb0 = 2 * ((g + 1) & 1);
            const bool more = g + 1 < 4;
            const f16x8 (&f)[4] = (g & 1) ? fb : fa;
            f16x8 (&n)[4] = (g & 1) ? fa : fb;
            const f16x8 pf = c4 == 2 ? pf2 : pf3, sf = c4 == 2 ? sf2 : sf3;
            int oa0, ob0, oa1, ob1;
            swz_trans_offsets<D>(nc4 * 16, ndb0 * 32, lane, oa0, ob0);
            swz_trans_offsets<D>(nc4 * 16, (ndb0 + 1) * 32, lane, oa1, ob1);
            __builtin_amdgcn_sched_barrier(0);
            acc_mfma16(dvacc[db0], f[0], pf);
            __builtin_amdgcn_sched_barrier(0);
            if (more) n[0] = swz_trans(Gt, oa0, ob0);
            __builtin_amdgcn_sched_barrier(0);
            acc_mfma16(dkacc[db0], f[1], sf);
            __builtin_amdgcn_sched_barrier(0);
            if (more) n[1] = swz_trans(Qt, oa0, ob0);
            __builtin_amdgcn_sched_barrier(0);
            acc_mfma16(dvacc[db0 + 1], f[2], pf);
            __builtin_amdgcn_sched_barrier(0);
            if (more) n[2] = swz_trans(Gt, oa1, ob1);
            __builtin_amdgcn_sched_barrier(0);
            acc_mfma16(dkacc[db0 + 1], f[3], sf);
            __builtin_amdgcn_sched_barrier(0);
            if (more) n[3] = swz_trans(Qt, oa1, ob1);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    auto tile = [&](int buf, auto masked_tag, int jt_next, int buf_next) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        if constexpr (D == 128 && !MASKED) { tile_d128(buf, masked_tag, jt_next, buf_next); return; }
        const uint16_t* Qt = q_tile(buf);
        const uint16_t* Gt = g_tile(buf);
        const uint16_t* At = aux_tile(buf);
        const uint32_t* qpos_t = qpos_tile(buf);
        f32x16 sacc[2], pacc[2];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            const f16x8 ax = as_f16x8(*reinterpret_cast<const uint4*>(&At[(qb * 32 + l32) * 8]));
            sacc[qb] = mfma16(ax, sub_lse, zero16());
            pacc[qb] = mfma16(ax, sub_delta, zero16());
        }
        if (D == 128) {
            // one wavefront per SIMD: nobody else hides its LDS latency, so the row fragments of a contraction
            // step are requested a full step (four matrix instructions) before they are used
            f16x8 fq[2][2], fg[2][2];
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                fq[0][qb] = swz_rows<D>(Qt, qb * 32 + l32, h * 8);
                fg[0][qb] = swz_rows<D>(Gt, qb * 32 + l32, h * 8);
            }
#pragma unroll
            for (int kk = 0; kk < D / 16; ++kk) {
                if (kk + 1 < D / 16) {
#pragma unroll
                    for (int qb = 0; qb < 2; ++qb) {
                        fq[(kk + 1) & 1][qb] = swz_rows<D>(Qt, qb * 32 + l32, (kk + 1) * 16 + h * 8);
                        fg[(kk + 1) & 1][qb] = swz_rows<D>(Gt, qb * 32 + l32, (kk + 1) * 16 + h * 8);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int qb = 0; qb < 2; ++qb) {
                    sacc[qb] = mfma16(fq[kk & 1][qb], kf[kk], sacc[qb]);
                    pacc[qb] = mfma16(fg[kk & 1][qb], vf[kk], pacc[qb]);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
#pragma unroll
            for (int kk = 0; kk < D / 16; ++kk)
#pragma unroll
                for (int qb = 0; qb < 2; ++qb) {
                    sacc[qb] = mfma16(swz_rows<D>(Qt, qb * 32 + l32, kk * 16 + h * 8), kf[kk], sacc[qb]);
                    pacc[qb] = mfma16(swz_rows<D>(Gt, qb * 32 + l32, kk * 16 + h * 8), vf[kk], pacc[qb]);
                }
        }

#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                uint32_t qpa[4] = {0u, 0u, 0u, 0u};
                if (MASKED) {
                    const uint4 qp = *reinterpret_cast<const uint4*>(&qpos_t[qb * 32 + 8 * g + 4 * h]);
                    qpa[0] = qp.x; qpa[1] = qp.y; qpa[2] = qp.z; qpa[3] = qp.w;
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float p = fast_exp2(sacc[qb][4 * g + e] * cexp);
                    if (MASKED) { if (qpa[e] - klo > kspan) p = 0.f; }     // bucket and causal test on the sort keys
                    sacc[qb][4 * g + e] = p;
                }
            }

#pragma unroll
        for (int c4 = 0; c4 < 4; ++c4) {
            const f16x8 pf = pack_chunk(sacc[c4 >> 1], c4 & 1);
            const f16x8 sf = pf * pack_chunk(pacc[c4 >> 1], c4 & 1);   // dS = P (dP - D), two elements per instruction
#pragma unroll
            for (int db = 0; db < D / 32; ++db) {
                int oa, ob;
                swz_trans_offsets<D>(c4 * 16, db * 32, lane, oa, ob);
                if (D == 128) {   // 128 accumulator registers: kept out of the architectural VGPRs
                    acc_mfma16(dvacc[db], swz_trans(Gt, oa, ob), pf);
                    acc_mfma16(dkacc[db], swz_trans(Qt, oa, ob), sf);
                } else {
                    dvacc[db] = mfma16(swz_trans(Gt, oa, ob), pf, dvacc[db]);
                    dkacc[db] = mfma16(swz_trans(Qt, oa, ob), sf, dkacc[db]);
                }
            }
        }
    };

#pragma unroll
    for (int u = 0; u < NBUF - 1; ++u) issue(u, u);
    // one step: wait for this wavefront's share of tile jt, barrier (everyone's share has landed and
    // everyone has left tile jt - 1), refill that tile's buffer, compute
    int cur = 0;
    auto step = [&](int jt, auto masked_tag) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        wait_async<LOADS_PER_TILE * (NBUF - 2)>();
        lds_barrier();
        const int refill = cur == 0 ? NBUF - 1 : cur - 1;
        constexpr bool SPREAD = D == 128 && !MASKED;   // the hand-ordered tile issues the loads itself, between its groups
        if (!SPREAD) issue(jt + NBUF - 1, refill);
        // sort keys ascend along the queries of an item: a tile that lies entirely below or entirely
        // above what may see the keys of this wavefront contributes nothing to it
        bool skip = false;
        if (MASKED) {
            const int last = min(BM, q_count - jt * BM) - 1;
            skip = (uint32_t)__builtin_amdgcn_readfirstlane(qpos_tile(cur)[last]) < klo_wave ||
                   (uint32_t)__builtin_amdgcn_readfirstlane(qpos_tile(cur)[0]) > khi_wave;
        }
        if (!skip) tile(cur, masked_tag, jt + NBUF - 1, refill);
        cur = cur == NBUF - 1 ? 0 : cur + 1;
    };
    int jt = 0;
    for (; jt < n_masked; ++jt) step(jt, std::true_type{});
    for (; jt < n_tiles; ++jt) step(jt, std::false_type{});
    wait_async<0>();   // nothing may still be landing in LDS when the wavefront ends
    if constexpr (D == 128) acc_mfma_drain(dvacc[0], dvacc[1], dvacc[2], dvacc[3], dkacc[0], dkacc[1], dkacc[2], dkacc[3]);
    if (kvalid) {
        const float us = inv_scale[s];
        const float sk = tau * us;   // dK = tau dS^T Q
        float* dkp = dk + (seg + kpos) * D + 4 * h;
        float* dvp = dv + (seg + kpos) * D + 4 * h;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                *reinterpret_cast<float4*>(dkp + db * 32 + 8 * g) =
                    make_float4(dkacc[db][4 * g] * sk, dkacc[db][4 * g + 1] * sk, dkacc[db][4 * g + 2] * sk, dkacc[db][4 * g + 3] * sk);
                *reinterpret_cast<float4*>(dvp + db * 32 + 8 * g) =
                    make_float4(dvacc[db][4 * g] * us, dvacc[db][4 * g + 1] * us, dvacc[db][4 * g + 2] * us, dvacc[db][4 * g + 3] * us);
            }
    }
}

template <int D>
static int launch_dkdv_t(const void* q, const void* k, const void* v, const void* do_perm,
                         const void* aux_perm, const float* inv_scale,
                         const uint32_t* q_key, const uint32_t* k_key, const int32_t* work, int n_work, int S,
                         int T, float tau, int strict, float* dk, float* dv, const int32_t* n_keep_k, hipStream_t st)
{
    const size_t smem = (size_t)DkdvRing<D>::NBUF * DkdvRing<D>::BUF_BYTES;
    static std::atomic<unsigned long long> lds_allowed{0};
    { const int rc_ = allow_dynamic_lds(reinterpret_cast<const void*>(&attn_bwd_dkdv_f16_kernel<D>), (int)smem, lds_allowed); if (rc_ != SCFA_OK) return rc_; }
    dim3 grid((unsigned)((size_t)S * n_work)), block(256);
    hipLaunchKernelGGL(attn_bwd_dkdv_f16_kernel<D>, grid, block, smem, st, (const uint16_t*)q, (const uint16_t*)k,
                       (const uint16_t*)v, (const uint16_t*)do_perm, (const uint16_t*)aux_perm, inv_scale, q_key, k_key,
                       work, n_work, S, T, tau, strict, dk, dv, n_keep_k);
    SCFA_HIP_TRY(hipGetLastError());
    return SCFA_OK;
}

template <int D>
static int occupancy_dkdv_t(int* out)
{
    const size_t smem = (size_t)DkdvRing<D>::NBUF * DkdvRing<D>::BUF_BYTES;
    SCFA_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_bwd_dkdv_f16_kernel<D>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    SCFA_HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(out, reinterpret_cast<const void*>(&attn_bwd_dkdv_f16_kernel<D>), 256, smem));
    return SCFA_OK;
}

// workgroups of the dK/dV kernel one CU holds at once
int occupancy_attn_bwd_dkdv_bf16(int d, int* out)
{
    return d == 64 ? occupancy_dkdv_t<64>(out) : d == 128 ? occupancy_dkdv_t<128>(out) : SCFA_EUNSUPPORTED;
}

int launch_attn_bwd_dkdv_bf16(const void* q, const void* k, const void* v, const void* do_perm,
                              const void* aux_perm, const float* inv_scale,
                              const uint32_t* q_key, const uint32_t* k_key, const int32_t* bwd_work, int n_bwd,
                              int S, int T, int d, float tau, int strict, float* dk, float* dv, const int32_t* n_keep_k,
                              hipStream_t st)
{
    ProfScope prof(SCFA_K_BWD_DKDV, st);
    if (d == 64)
        return launch_dkdv_t<64>(q, k, v, do_perm, aux_perm, inv_scale, q_key, k_key, bwd_work, n_bwd, S, T, tau, strict, dk, dv, n_keep_k, st);
    if (d == 128)
        return launch_dkdv_t<128>(q, k, v, do_perm, aux_perm, inv_scale, q_key, k_key, bwd_work, n_bwd, S, T, tau, strict, dk, dv, n_keep_k, st);
    return SCFA_EUNSUPPORTED;
}

// ===========================================================================
// dQ: same walk as the forward (a workgroup owns 128 queries of one bucket, 32 per
// wavefront in the lanes; keys 64 at a time).  Per tile:
//   X^T = K Q'^T - LSE log2 e, dP'^T = V dO^T - D (keys x queries; the accumulators start
//   from the per-lane constants), P^T = 2^X^T, dS^T = P^T dP'^T, dQ^T += K^T dS^T
// ===========================================================================
// LDS ring of the dQ kernel: K tile, V tile and key positions per buffer, filled asynchronously
// NBUF - 1 tiles ahead (the forward kernel's scheme)
template <int D>
struct DqRing {
    static constexpr int BN = FWD_TILE_N;
    static constexpr int TILE_ELEMS = BN * D;
    static constexpr int BUF_BYTES = TILE_ELEMS * 4 + BN * 4;
    static constexpr int NBUF = D == 64 ? 3 : 2;
};

// Two wavefronts per SIMD are asked for explicitly: at d = 128 the register allocator would otherwise take a
// few AccVGPRs beyond 256 registers and halve the occupancy.
template <int D>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void attn_bwd_dq_f16_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const uint16_t* __restrict__ do_perm, const float* __restrict__ lse_perm,
    const float* __restrict__ delta_perm, const float* __restrict__ inv_scale,
    const uint32_t* __restrict__ q_key, const uint32_t* __restrict__ k_key,
    const int32_t* __restrict__ work, int n_work, int S, int T, float tau, int strict, float* __restrict__ dq,
    const int32_t* __restrict__ n_keep_q)
{
    constexpr int BN = FWD_TILE_N;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    constexpr int NBUF = DqRing<D>::NBUF, BUF_BYTES = DqRing<D>::BUF_BYTES, TILE_ELEMS = DqRing<D>::TILE_ELEMS;
    constexpr int KPW = BN / 4;                                               // key positions loaded per wavefront
    constexpr int LOADS_PER_TILE = 2 * AsyncTile<D, BN, 256>::ROUNDS + 1;     // per wavefront
    auto k_tile = [&](int buf) { return reinterpret_cast<const uint16_t*>(smem_raw + buf * BUF_BYTES); };
    auto v_tile = [&](int buf) { return reinterpret_cast<const uint16_t*>(smem_raw + buf * BUF_BYTES + TILE_ELEMS * 2); };
    auto kpos_tile = [&](int buf) { return reinterpret_cast<uint32_t*>(smem_raw + buf * BUF_BYTES + TILE_ELEMS * 4); };
    const uint32_t lds0 = lds_address(smem_raw);

    const int s = blockIdx.x % S;
    const int w = blockIdx.x / S;
    const int32_t* it = work + ((size_t)s * n_work + w) * WORK_STRIDE;
    const int q_begin = it[W_QBEGIN], q_count = it[W_QCOUNT];
    const int k_begin = it[W_KBEGIN], k_count = it[W_KCOUNT], k_nomask = it[W_KNOMASK];
    if (q_count <= 0) {   // no work: only the share of the dropped rows (n_keep_q: QK-dropping, else null)
        if (n_keep_q) zero_dropped_rows<D>(q_key + (size_t)s * T, n_keep_q[s], T, w, n_work, dq, nullptr, (size_t)s * T);
        return;
    }

    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, l32 = lane & 31, h = lane >> 5;
    const size_t seg = (size_t)s * T;
    if (n_keep_q) zero_dropped_rows<D>(q_key + seg, n_keep_q[s], T, w, n_work, dq, nullptr, seg);
    const int qrow = wave * 32 + l32;
    const bool qvalid = qrow < q_count;
    const int qr = min(qrow, q_count - 1);              // rows past the end repeat the last one; never written
    const uint32_t qkey = q_key[seg + q_begin + qr];
    const int qpos = (int)(qkey & KEY_POS_MASK);
    // a key is allowed iff (its sort key - qlo) <= qspan: same bucket, position <= the query's (< if strict)
    const bool some = qvalid && qpos - strict >= 0;
    const uint32_t qlo = some ? (qkey & ~KEY_POS_MASK) : KEY_NEVER;
    const uint32_t qspan = some ? (uint32_t)(qpos - strict) : 0u;
    const float cexp = tau * LOG2E;   // scores are raw <q, k> sums: P = 2^(cexp s - LSE log2 e), one fma per element
    const float lse_ld = lse_perm[seg + q_begin + qr];
    const float lse2 = (qvalid && lse_ld != -INFINITY) ? fmaf(lse_ld, LOG2E, -RTZ_BIAS_LOG2) : INFINITY;
    const float delta = delta_perm[seg + q_begin + qr];

    f16x8 qf[D / 16], gf[D / 16];
    {
        const uint16_t* qp = q + (seg + q_begin + qr) * D + h * 8;
        const uint16_t* gp = do_perm + (seg + q_begin + qr) * D + h * 8;
#pragma unroll
        for (int kk = 0; kk < D / 16; ++kk) {
            qf[kk] = as_f16x8(*reinterpret_cast<const uint4*>(qp + kk * 16));
            gf[kk] = as_f16x8(*reinterpret_cast<const uint4*>(gp + kk * 16));
        }
#pragma unroll
        for (int kk = 0; kk < D / 16; ++kk) { touch(qf[kk]); touch(gf[kk]); }
    }

    f32x16 dqacc[D / 32], p_start;   // loop-invariant accumulator start of dP: -D
#pragma unroll
    for (int db = 0; db < D / 32; ++db) dqacc[db] = zero16();
#pragma unroll
    for (int i = 0; i < 16; ++i) p_start[i] = -delta;

    const int n_tiles = (k_count + BN - 1) / BN;
    const int n_free = min(k_nomask / BN, n_tiles);
    // the sort keys any query of this wavefront may attend to lie in [qlo_wave, qhi_wave]
    uint32_t qlo_wave = some ? qlo : 0xffffffffu, qhi_wave = some ? qlo + qspan : 0u;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        qlo_wave = min(qlo_wave, (uint32_t)__shfl_xor((int)qlo_wave, off));
        qhi_wave = max(qhi_wave, (uint32_t)__shfl_xor((int)qhi_wave, off));
    }
    qlo_wave = __builtin_amdgcn_readfirstlane(qlo_wave);
    qhi_wave = __builtin_amdgcn_readfirstlane(qhi_wave);

    AsyncTile<D, BN, 256> loader;
    loader.init();
    const u32x4 k_desc = make_desc(k + (seg + k_begin) * D, (uint32_t)k_count * D * 2);
    const u32x4 v_desc = make_desc(v + (seg + k_begin) * D, (uint32_t)k_count * D * 2);
    const u32x4 p_desc = make_desc(k_key + seg + k_begin, (uint32_t)k_count * 4);
    // every wavefront issues the same number of loads per tile, so one vmcnt threshold serves all;
    // tiles past the end read zeros into a buffer nobody uses
    auto issue = [&](int jt, int buf) {
        const uint32_t base = lds0 + (uint32_t)(buf * BUF_BYTES);
        loader.load(k_desc, jt * loader.TILE_BYTES, base);
        loader.load(v_desc, jt * loader.TILE_BYTES, base + TILE_ELEMS * 2);
        if (lane < KPW)
            async_load4(p_desc, __builtin_amdgcn_readfirstlane(base + TILE_ELEMS * 4 + wave * KPW * 4),
                        (wave * KPW + lane) * 4, jt * BN * 4);
    };

    auto tile = [&](int buf, auto masked_tag) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        const uint16_t* Kt = k_tile(buf);
        const uint16_t* Vt = v_tile(buf);
        const uint32_t* kpos_t = kpos_tile(buf);
        // KBS 32-key blocks of the tile are in flight at once: both at d = 64; one at a time at
        // d = 128, where two sets of score accumulators would push the kernel past 256 registers
        // and down to one wavefront per SIMD
        constexpr int KBS = D == 64 ? 2 : 1;
#pragma unroll
        for (int k0 = 0; k0 < 2; k0 += KBS) {
            f32x16 sacc[KBS], pacc[KBS];
#pragma unroll
            for (int kb = 0; kb < KBS; ++kb) {
                sacc[kb] = zero16();
                if (KBS == 2) {
                    pacc[kb] = p_start;                         // read as the C operand of the first MFMA: no moves
                } else {                                        // registers are scarcer than moves at d = 128
                    float p0 = p_start[0];
                    asm volatile("" : "+v"(p0));                // not a loop invariant: splat here, every time
#pragma unroll
                    for (int i = 0; i < 16; ++i) pacc[kb][i] = p0;
                }
            }
            if (KBS == 1) {
                // two wavefronts per SIMD do not hide the LDS latency of a read issued at its use: the row
                // fragments of a contraction step are requested one step (two matrix instructions) ahead
                f16x8 fk[2], fv[2];
                fk[0] = swz_rows<D>(Kt, k0 * 32 + l32, h * 8);
                fv[0] = swz_rows<D>(Vt, k0 * 32 + l32, h * 8);
#pragma unroll
                for (int kk = 0; kk < D / 16; ++kk) {
                    if (kk + 1 < D / 16) {
                        fk[(kk + 1) & 1] = swz_rows<D>(Kt, k0 * 32 + l32, (kk + 1) * 16 + h * 8);
                        fv[(kk + 1) & 1] = swz_rows<D>(Vt, k0 * 32 + l32, (kk + 1) * 16 + h * 8);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    sacc[0] = mfma16(fk[kk & 1], qf[kk], sacc[0]);
                    pacc[0] = mfma16(fv[kk & 1], gf[kk], pacc[0]);
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
#pragma unroll
                for (int kk = 0; kk < D / 16; ++kk)
#pragma unroll
                    for (int kb = 0; kb < KBS; ++kb) {
                        sacc[kb] = mfma16(swz_rows<D>(Kt, (k0 + kb) * 32 + l32, kk * 16 + h * 8), qf[kk], sacc[kb]);
                        pacc[kb] = mfma16(swz_rows<D>(Vt, (k0 + kb) * 32 + l32, kk * 16 + h * 8), gf[kk], pacc[kb]);
                    }
            }

            // d = 128: the transposed K fragments of the first 16-key chunk are requested before the
            // exponentials, those of the second chunk while the first chunk's products run
            f16x8 tk[2][KBS == 1 ? D / 32 : 1];
            if (KBS == 1) {
#pragma unroll
                for (int db = 0; db < D / 32; ++db) {
                    int oa, ob;
                    swz_trans_offsets<D>(2 * k0 * 16, db * 32, lane, oa, ob);
                    tk[0][db] = swz_trans(Kt, oa, ob);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int kb = 0; kb < KBS; ++kb)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    uint32_t kpa[4] = {0u, 0u, 0u, 0u};
                    if (MASKED) {
                        const uint4 kp = *reinterpret_cast<const uint4*>(&kpos_t[(k0 + kb) * 32 + 8 * g + 4 * h]);
                        kpa[0] = kp.x; kpa[1] = kp.y; kpa[2] = kp.z; kpa[3] = kp.w;
                    }
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        float p = fast_exp2(fmaf(sacc[kb][4 * g + e], cexp, -lse2));
                        if (MASKED) { if (kpa[e] - qlo > qspan) p = 0.f; }     // bucket and causal test on the sort keys
                        pacc[kb][4 * g + e] = p * pacc[kb][4 * g + e];
                    }
                }

            if (KBS == 1) {
                const f16x8 sf0 = pack_chunk(pacc[0], 0), sf1 = pack_chunk(pacc[0], 1);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int db = 0; db < D / 32; ++db) {
                    int oa, ob;
                    swz_trans_offsets<D>((2 * k0 + 1) * 16, db * 32, lane, oa, ob);
                    tk[1][db] = swz_trans(Kt, oa, ob);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int db = 0; db < D / 32; ++db) dqacc[db] = mfma16(tk[0][db], sf0, dqacc[db]);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int db = 0; db < D / 32; ++db) dqacc[db] = mfma16(tk[1][db], sf1, dqacc[db]);
                __builtin_amdgcn_sched_barrier(0);   // keep the two blocks apart
            } else {
#pragma unroll
                for (int c = 0; c < 2 * KBS; ++c) {
                    const int c4 = 2 * k0 + c;       // 16-key chunk of the tile
                    const f16x8 sf = pack_chunk(pacc[c >> 1], c & 1);
#pragma unroll
                    for (int db = 0; db < D / 32; ++db) {
                        int oa, ob;
                        swz_trans_offsets<D>(c4 * 16, db * 32, lane, oa, ob);
                        dqacc[db] = mfma16(swz_trans(Kt, oa, ob), sf, dqacc[db]);
                    }
                }
            }
        }
    };

#pragma unroll
    for (int u = 0; u < NBUF - 1; ++u) issue(u, u);
    // one step: wait for this wavefront's share of tile jt, mark keys past the end of a ragged
    // tile (always a masked tile), barrier, refill the buffer everyone has just left, compute
    int cur = 0;
    auto step = [&](int jt, auto masked_tag) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        wait_async<LOADS_PER_TILE * (NBUF - 2)>();
        if (MASKED && lane < KPW) {
            const int key = jt * BN + wave * KPW + lane;
            if (key >= k_count) kpos_tile(cur)[wave * KPW + lane] = KEY_PAST_END;   // never allowed
        }
        lds_barrier();
        const int refill = cur == 0 ? NBUF - 1 : cur - 1;    // the buffer of tile jt - 1
        issue(jt + NBUF - 1, refill);
        // sort keys ascend along the keys of an item: a tile that lies entirely above or entirely
        // below what the queries of this wavefront may attend to contributes nothing to it
        bool skip = false;
        if (MASKED)
            skip = (uint32_t)__builtin_amdgcn_readfirstlane(kpos_tile(cur)[0]) > qhi_wave ||
                   (uint32_t)__builtin_amdgcn_readfirstlane(kpos_tile(cur)[BN - 1]) < qlo_wave;
        if (!skip) tile(cur, masked_tag);
        cur = cur == NBUF - 1 ? 0 : cur + 1;
    };
    int jt = 0;
    for (; jt < n_free; ++jt) step(jt, std::false_type{});
    for (; jt < n_tiles; ++jt) step(jt, std::true_type{});
    wait_async<0>();   // nothing may still be landing in LDS when the wavefront ends

    if (qvalid) {
        const float sq = tau * inv_scale[s];
        float* dqp = dq + (seg + qpos) * D + 4 * h;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g)
                *reinterpret_cast<float4*>(dqp + db * 32 + 8 * g) =
                    make_float4(dqacc[db][4 * g] * sq, dqacc[db][4 * g + 1] * sq, dqacc[db][4 * g + 2] * sq, dqacc[db][4 * g + 3] * sq);
    }
}

template <int D>
static int launch_dq_t(const void* q, const void* k, const void* v, const void* do_perm,
                       const float* lse_perm, const float* delta_perm, const float* inv_scale,
                       const uint32_t* q_key, const uint32_t* k_key, const int32_t* work, int n_work, int S, int T,
                       float tau, int strict, float* dq, const int32_t* n_keep_q, hipStream_t st)
{
    const size_t smem = (size_t)DqRing<D>::NBUF * DqRing<D>::BUF_BYTES;
    static std::atomic<unsigned long long> lds_allowed{0};
    { const int rc_ = allow_dynamic_lds(reinterpret_cast<const void*>(&attn_bwd_dq_f16_kernel<D>), (int)smem, lds_allowed); if (rc_ != SCFA_OK) return rc_; }
    dim3 grid((unsigned)((size_t)S * n_work)), block(256);
    hipLaunchKernelGGL(attn_bwd_dq_f16_kernel<D>, grid, block, smem, st, (const uint16_t*)q, (const uint16_t*)k,
                       (const uint16_t*)v, (const uint16_t*)do_perm, lse_perm, delta_perm, inv_scale, q_key, k_key,
                       work, n_work, S, T, tau, strict, dq, n_keep_q);
    SCFA_HIP_TRY(hipGetLastError());
    return SCFA_OK;
}

template <int D>
static int occupancy_dq_t(int* out)
{
    const size_t smem = (size_t)DqRing<D>::NBUF * DqRing<D>::BUF_BYTES;
    SCFA_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_bwd_dq_f16_kernel<D>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    SCFA_HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(out, reinterpret_cast<const void*>(&attn_bwd_dq_f16_kernel<D>), 256, smem));
    return SCFA_OK;
}

// workgroups of the dQ kernel one CU holds at once
int occupancy_attn_bwd_dq_bf16(int d, int* out)
{
    return d == 64 ? occupancy_dq_t<64>(out) : d == 128 ? occupancy_dq_t<128>(out) : SCFA_EUNSUPPORTED;
}

int launch_attn_bwd_dq_bf16(const void* q, const void* k, const void* v, const void* do_perm,
                            const float* lse_perm, const float* delta_perm, const float* inv_scale,
                            const uint32_t* q_key, const uint32_t* k_key, const int32_t* fwd_work, int n_fwd,
                            int S, int T, int d, float tau, int strict, float* dq, const int32_t* n_keep_q, hipStream_t st)
{
    ProfScope prof(SCFA_K_BWD_DQ, st);
    if (d == 64)
        return launch_dq_t<64>(q, k, v, do_perm, lse_perm, delta_perm, inv_scale, q_key, k_key, fwd_work, n_fwd, S, T, tau, strict, dq, n_keep_q, st);
    if (d == 128)
        return launch_dq_t<128>(q, k, v, do_perm, lse_perm, delta_perm, inv_scale, q_key, k_key, fwd_work, n_fwd, S, T, tau, strict, dq, n_keep_q, st);
    return SCFA_EUNSUPPORTED;
}

}  // namespace scfa

