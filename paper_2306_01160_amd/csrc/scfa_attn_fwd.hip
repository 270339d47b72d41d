// Forward attention over the work list, fp16 compute format, fp32 accumulation.
//
// A workgroup owns one work item: up to 128 query rows of one bucket and the range of keys
// of the same bucket that causality can let through, or all rows of a few small buckets on
// both sides (scfa_block_ranges).  Keys are walked 64 at a time; tiles the schedule proved
// mask-free come first and run without any test, the remaining tiles test bucket and
// causality at once on the rows' sort keys, bucket << 24 | original position (paper
// Sec. 3.1 / 3.2: a local mask from the index and bucket vectors).  Sort keys ascend along
// an item's keys, so a wavefront also skips a masked tile that lies entirely outside the
// key range its own 32 queries can match.
//
// A wavefront keeps its query rows in the lanes: S^T = K Q^T puts one query per lane
// (column) and 16 keys per accumulator block in its registers, so the softmax
// statistics are per-lane scalars and S^T's accumulator layout is already the
// B-operand layout of O^T += V^T P^T.  V^T comes from the row-major V tile through
// transposing LDS reads.
//
// K / V tiles and the key positions travel global memory -> LDS asynchronously (no
// registers, no LDS stores), NBUF - 1 tiles ahead of the one being computed, into a ring of
// NBUF swizzled buffers; one workgroup barrier per tile both publishes the tile that has
// landed and retires the buffer that is refilled next.
//
// The permuted queries and keys are the inputs' own values (bf16 -> fp16 is exact), so the
// contraction yields <q, k> exactly up to the fp32 accumulation, and the softmax scale enters
// as one fused multiply-add per element, p = 2^(tau log2(e) (<q, k> - m) + bias): the
// logsumexp this kernel hands out carries no rounding of the operands.  (The backward kernels
// fold the scale into their register-resident operand instead and save that instruction: a
// 2^-12 relative error per element of the recomputed scores does not matter to the gradients,
// but it would be the largest term of the logsumexp error.)
//
// Online softmax (paper App. B.1, running maximum and sum, NaN-safe for fully masked
// rows): the accumulator is un-normalised and divided by the sum once at the end.  The
// reference maximum m (of the raw sums) is only raised when some row's tile maximum exceeds
// it by more than LAZY_LOG2 base-2 units (then the accumulator and the sum are rescaled by
// 2^(c (m_old - m_new)), c = tau log2(e)); between raises P = 2^(c (s - m)) may exceed 1 but
// stays inside the fp16 range.  Once every
// row of a wavefront has a finite reference, the tile maximum is not even computed: the
// row sum of the packed probabilities, needed anyway, exceeds 2^15 in some lane whenever
// a probability has left the fp16 range (packing truncates to at most 65504), and only
// then is the tile redone with its maximum as the new reference.  Because
// m changes rarely, -m is kept splatted over an accumulator block and the score
// contraction starts from it: the matrix core delivers s - m and the only per-element
// vector work left is the scaling, the exponential, the packing and the row sum.  A row that never
// sees an allowed key keeps m = -inf and l = 0; its exponent base is 0 (the paper's
// replacement of -inf by 0), every p is 2^(-inf) = 0, and it is written as zeros with
// LSE = -inf.
#include "scfa_common.hpp"
#include "scfa_mma.hpp"

#include <math.h>
#include <type_traits>

namespace scfa {

constexpr float LAZY_LOG2 = 6.0f;
constexpr float SUM_LIMIT = 32768.f;   // a lane's tile sum above this may hide a probability beyond the fp16 range

// LDS ring of the forward kernel: as many buffers as three resident workgroups allow
template <int D>
struct FwdRing {
    static constexpr int BUF_BYTES = FWD_TILE_N * D * 4 + FWD_TILE_N * 4;
    static constexpr int NBUF = D == 64 ? 3 : 2;
};

// QK-dropping: the output rows of dropped queries are zeros and their LSE is -inf.  Every workgroup of the forward kernel, the
// ones without work included, writes a strided share of its segment's dropped rows next to its own stores (a launch of its own
// for them ran with nothing beside it).  key_seg: the segment's query index vector, dropped positions from n_keep on.
template <int D, int THREADS>
__device__ __forceinline__ void fill_dropped_rows(const uint32_t* __restrict__ key_seg, int n_keep, int T, int w, int n_wg,
                                                  uint16_t* __restrict__ o, float* __restrict__ lse, size_t seg)
{
    constexpr int CPR = D / 8, R = THREADS / CPR;   // 16-byte pieces per bf16 row, rows per pass
    const int sub = (int)threadIdx.x / CPR, c = (int)threadIdx.x % CPR;
    for (long long r = (long long)n_keep + (long long)w * R + sub; r < T; r += (long long)n_wg * R) {
        const size_t pos = seg + (key_seg[r] & KEY_POS_MASK);
        reinterpret_cast<uint4*>(o + pos * D)[c] = make_uint4(0u, 0u, 0u, 0u);
        if (c == 0) lse[pos] = -INFINITY;
    }
}

template <int D, int NW, int QB>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(D == 64 ? 3 : 2))) void attn_fwd_f16_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const uint32_t* __restrict__ q_key, const uint32_t* __restrict__ k_key,
    const int32_t* __restrict__ work, int n_work, int S, int T, float tau, int strict,
    uint16_t* __restrict__ o, float* __restrict__ lse, uint16_t* __restrict__ o_f16, const int32_t* __restrict__ n_keep_q)
{
    static_assert(NW * QB * 32 == FWD_TILE_M, "workgroup must cover the forward query tile");
    const float cexp = tau * LOG2E;   // scores are raw <q, k> sums; the exponent of every probability is cexp * (sum - m)
    constexpr int BN = FWD_TILE_N;
    constexpr int THREADS = NW * 64;
    constexpr int NBUF = FwdRing<D>::NBUF;            // LDS ring; NBUF - 1 tiles are in flight
    constexpr int TILE_ELEMS = BN * D;
    constexpr int BUF_BYTES = FwdRing<D>::BUF_BYTES;  // K tile, V tile, key positions
    constexpr int LOADS_PER_TILE = 2 * AsyncTile<D, BN, THREADS>::ROUNDS + 1;   // per wavefront
    constexpr int KPW = BN / NW;                      // key positions loaded per wavefront
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    auto k_tile = [&](int buf) { return reinterpret_cast<const uint16_t*>(smem_raw + buf * BUF_BYTES); };
    auto v_tile = [&](int buf) { return reinterpret_cast<const uint16_t*>(smem_raw + buf * BUF_BYTES + TILE_ELEMS * 2); };
    auto kpos_tile = [&](int buf) { return reinterpret_cast<uint32_t*>(smem_raw + buf * BUF_BYTES + TILE_ELEMS * 4); };
    const uint32_t lds0 = lds_address(smem_raw);

    // consecutive workgroups take the same work rank of consecutive segments: the longest
    // items of every segment are dispatched first, and when S is a multiple of 8 a segment
    // stays on one XCD (its K/V stay in that XCD's L2).
    const int s = blockIdx.x % S;
    const int w = blockIdx.x / S;
    const int32_t* it = work + ((size_t)s * n_work + w) * WORK_STRIDE;
    const int q_begin = it[W_QBEGIN], q_count = it[W_QCOUNT];
    const int k_begin = it[W_KBEGIN], k_count = it[W_KCOUNT], k_nomask = it[W_KNOMASK];
    if (n_keep_q) fill_dropped_rows<D, THREADS>(q_key + (size_t)s * T, n_keep_q[s], T, w, n_work, o, lse, (size_t)s * T);
    if (q_count <= 0) return;

    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, l32 = lane & 31, h = lane >> 5;
    const size_t seg = (size_t)s * T;

    int qrow[QB], qpos[QB];
    // a key is allowed iff (its sort key - qlo) <= qspan: same bucket, position <= the query's (< if strict)
    uint32_t qlo[QB], qspan[QB];
    bool qvalid[QB];
    f16x8 qf[QB][D / 16];
#pragma unroll
    for (int b = 0; b < QB; ++b) {
        qrow[b] = (wave * QB + b) * 32 + l32;
        qvalid[b] = qrow[b] < q_count;
        const int qr = min(qrow[b], q_count - 1);          // rows past the end repeat the last one
        const uint32_t qk_ = q_key[seg + q_begin + qr];
        const int qp_ = (int)(qk_ & KEY_POS_MASK);
        qpos[b] = qvalid[b] ? qp_ : -1;
        const bool some = qvalid[b] && qp_ - strict >= 0;
        qlo[b] = some ? (qk_ & ~KEY_POS_MASK) : KEY_NEVER;   // KEY_NEVER, span 0: every key is masked
        qspan[b] = some ? (uint32_t)(qp_ - strict) : 0u;
        const uint16_t* qp = q + (seg + q_begin + qr) * D + h * 8;
#pragma unroll
        for (int kk = 0; kk < D / 16; ++kk) qf[b][kk] = as_f16x8(*reinterpret_cast<const uint4*>(qp + kk * 16));
    }
#pragma unroll
    for (int b = 0; b < QB; ++b)
#pragma unroll
        for (int kk = 0; kk < D / 16; ++kk) touch(qf[b][kk]);   // loaded before the tile loop starts

    f32x16 oacc[QB][D / 32];
    f32x16 start[QB];                // -(finite reference maximum), in all 16 registers
    float m[QB], thr[QB], lsum[QB];  // reference maximum (raw <q, k> units), raise threshold on s - m, partial row sum
#pragma unroll
    for (int b = 0; b < QB; ++b) {
#pragma unroll
        for (int db = 0; db < D / 32; ++db) oacc[b][db] = zero16();
#pragma unroll
        for (int i = 0; i < 16; ++i) start[b][i] = 0.f;
        m[b] = -INFINITY; thr[b] = -INFINITY; lsum[b] = 0.f;   // the first finite score always raises
    }

    // the sort keys any query of this wavefront may attend to lie in [qlo_wave, qhi_wave]
    uint32_t qlo_wave = 0xffffffffu, qhi_wave = 0u;
#pragma unroll
    for (int b = 0; b < QB; ++b)
        if (qlo[b] != KEY_NEVER) { qlo_wave = min(qlo_wave, qlo[b]); qhi_wave = max(qhi_wave, qlo[b] + qspan[b]); }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        qlo_wave = min(qlo_wave, (uint32_t)__shfl_xor((int)qlo_wave, off));
        qhi_wave = max(qhi_wave, (uint32_t)__shfl_xor((int)qhi_wave, off));
    }
    qlo_wave = __builtin_amdgcn_readfirstlane(qlo_wave);
    qhi_wave = __builtin_amdgcn_readfirstlane(qhi_wave);

    const uint16_t* kbase = k + (seg + k_begin) * D;
    const uint16_t* vbase = v + (seg + k_begin) * D;
    const uint32_t* kib = k_key + seg + k_begin;
    const int n_tiles = (k_count + BN - 1) / BN;
    const int n_free = k_nomask / BN;            // leading tiles that need no mask

    AsyncTile<D, BN, THREADS> loader;
    loader.init();
    const u32x4 k_desc = make_desc(kbase, (uint32_t)k_count * D * 2);
    const u32x4 v_desc = make_desc(vbase, (uint32_t)k_count * D * 2);
    const u32x4 p_desc = make_desc(kib, (uint32_t)k_count * 4);
    // every wavefront issues the same number of loads per tile (BN / NW key positions each), so one
    // vmcnt threshold serves all; tiles past the end read zeros into a buffer nobody uses
    auto issue = [&](int jt, int buf) {
        const uint32_t base = lds0 + (uint32_t)(buf * BUF_BYTES);
        loader.load(k_desc, jt * loader.TILE_BYTES, base);
        loader.load(v_desc, jt * loader.TILE_BYTES, base + TILE_ELEMS * 2);
        if (lane < KPW)
            async_load4(p_desc, __builtin_amdgcn_readfirstlane(base + TILE_ELEMS * 4 + wave * KPW * 4),
                        (wave * KPW + lane) * 4, jt * BN * 4);
    };

    // lane-invariant offsets of the transposing V reads
    int v_off[4][D / 32][2];
#pragma unroll
    for (int c4 = 0; c4 < 4; ++c4)
#pragma unroll
        for (int db = 0; db < D / 32; ++db) swz_trans_offsets<D>(c4 * 16, db * 32, lane, v_off[c4][db][0], v_off[c4][db][1]);

    bool settled = false;   // every row of this wavefront has a finite reference maximum (wave-uniform)
    auto tile = [&](int buf, auto masked_tag) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        const uint16_t* Kt = k_tile(buf);
        const uint16_t* Vt = v_tile(buf);
        const uint32_t* kpos_t = kpos_tile(buf);
        // S^T = K Q^T - m : [key block kb][query block b]
        f32x16 sacc[2][QB];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int b = 0; b < QB; ++b) sacc[kb][b] = start[b];
        if (D == 128) {
            // two wavefronts per SIMD do not hide the LDS latency of a read issued at its use: the K row
            // fragments of a contraction step are requested one step ahead
            f16x8 fk[2][2];
            fk[0][0] = swz_rows<D>(Kt, l32, h * 8);
            fk[0][1] = swz_rows<D>(Kt, 32 + l32, h * 8);
#pragma unroll
            for (int kk = 0; kk < D / 16; ++kk) {
                if (kk + 1 < D / 16) {
                    fk[(kk + 1) & 1][0] = swz_rows<D>(Kt, l32, (kk + 1) * 16 + h * 8);
                    fk[(kk + 1) & 1][1] = swz_rows<D>(Kt, 32 + l32, (kk + 1) * 16 + h * 8);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int b = 0; b < QB; ++b) sacc[kb][b] = mfma16(fk[kk & 1][kb], qf[b][kk], sacc[kb][b]);
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
#pragma unroll
            for (int kk = 0; kk < D / 16; ++kk)
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    const f16x8 a = swz_rows<D>(Kt, kb * 32 + l32, kk * 16 + h * 8);
#pragma unroll
                    for (int b = 0; b < QB; ++b) sacc[kb][b] = mfma16(a, qf[b][kk], sacc[kb][b]);
                }
        }

        if (MASKED) {   // bucket and causal test in one range test on the sort keys
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const uint4 kp = *reinterpret_cast<const uint4*>(&kpos_t[kb * 32 + 8 * g + 4 * h]);
#pragma unroll
                    for (int b = 0; b < QB; ++b) {
                        if (kp.x - qlo[b] > qspan[b]) sacc[kb][b][4 * g + 0] = -INFINITY;
                        if (kp.y - qlo[b] > qspan[b]) sacc[kb][b][4 * g + 1] = -INFINITY;
                        if (kp.z - qlo[b] > qspan[b]) sacc[kb][b][4 * g + 2] = -INFINITY;
                        if (kp.w - qlo[b] > qspan[b]) sacc[kb][b][4 * g + 3] = -INFINITY;
                    }
                }
        }

        // lane-local tile maximum per query; raise the reference only when needed
        auto raise_ref = [&]() {
        float mx[QB];
        bool raise = false;
#pragma unroll
        for (int b = 0; b < QB; ++b) {
            float a0 = sacc[0][b][0], a1 = sacc[1][b][0];
#pragma unroll
            for (int i = 1; i < 16; i += 2) {
                a0 = fmaxf(a0, fmaxf(sacc[0][b][i], sacc[0][b][(i + 1) & 15]));
                a1 = fmaxf(a1, fmaxf(sacc[1][b][i], sacc[1][b][(i + 1) & 15]));
            }
            mx[b] = fmaxf(a0, a1);
            raise |= mx[b] > thr[b];                    // -inf > -inf is false: no NaN is ever formed
        }
        if (__ballot(raise) != 0ull) {
#pragma unroll
            for (int b = 0; b < QB; ++b) {
                const float st_old = start[b][0];
                const float m_new = fmaxf(m[b], half_max(mx[b]) - st_old);   // tile maximum back in score units
                const float m_use = m_new == -INFINITY ? 0.f : m_new;
                float alpha = fast_exp2((m[b] - m_use) * cexp);                       // m = -inf -> 0
                asm volatile("" : "+v"(alpha));   // rare path: keeps the rescale from being speculated
                lsum[b] *= alpha;
#pragma unroll
                for (int db = 0; db < D / 32; ++db)
#pragma unroll
                    for (int i = 0; i < 16; ++i) oacc[b][db][i] *= alpha;
                const float st_new = -m_use;
                const float shift = st_new - st_old;    // scores of this tile move to the new reference
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) sacc[kb][b][i] += shift;
#pragma unroll
                for (int i = 0; i < 16; ++i) start[b][i] = st_new;
                m[b] = m_new;
                thr[b] = m_new == -INFINITY ? -INFINITY : LAZY_LOG2 / cexp;
            }
        }
        };

        // P = 2^(c (s - m) + bias), packed to fp16 (truncating: at most 65504, never inf); row sums from the
        // packed values
        f16x8 pf[QB][4];
        float lt[QB];
        auto exp_pack = [&]() {
#pragma unroll
        for (int b = 0; b < QB; ++b) {
            float l0 = 0.f, l1 = 0.f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int cc = 0; cc < 2; ++cc) {
                    uint32_t wv[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float p0 = fast_exp2(fmaf(sacc[kb][b][8 * cc + 2 * j], cexp, RTZ_BIAS_LOG2));
                        const float p1 = fast_exp2(fmaf(sacc[kb][b][8 * cc + 2 * j + 1], cexp, RTZ_BIAS_LOG2));
                        wv[j] = pack_f16(p0, p1);
                    }
                    l0 = add_pair(wv[0], l0); l1 = add_pair(wv[1], l1);
                    l0 = add_pair(wv[2], l0); l1 = add_pair(wv[3], l1);
                    pf[b][kb * 2 + cc] = as_f16x8(make_uint4(wv[0], wv[1], wv[2], wv[3]));
                }
            lt[b] = l0 + l1;
        }
        };

        // Until every row of the wavefront has a finite reference the tile maximum is taken first.
        // After that the maximum is not computed at all: the sum of the packed probabilities,
        // which is needed anyway, tells whether any of them left the fp16 range (a probability
        // beyond 2^15 makes its lane's sum exceed 2^15), and only then is the tile redone with
        // its maximum as the new reference.
        // (d = 64 only: at d = 128 the matrix cores, not the vector units, set the pace, and keeping
        // the scores alive for a possible second pass costs more than the maxima it saves)
        const bool by_sum = D == 64 && settled;
        if (!by_sum) {
            raise_ref();
            bool unset = false;
#pragma unroll
            for (int b = 0; b < QB; ++b) unset |= thr[b] == -INFINITY;
            settled = __ballot(unset) == 0ull;
        }
        exp_pack();
        if (by_sum) {
            bool big = false;
#pragma unroll
            for (int b = 0; b < QB; ++b) big |= lt[b] > SUM_LIMIT;
            if (__ballot(big) != 0ull) { raise_ref(); exp_pack(); }
        }
#pragma unroll
        for (int b = 0; b < QB; ++b) lsum[b] += lt[b];

        // O^T += V^T P^T
        if (D == 128) {   // the V^T fragments of a 16-key chunk are requested while the previous chunk's products run
            f16x8 fv[2][D / 32];
#pragma unroll
            for (int db = 0; db < D / 32; ++db) fv[0][db] = swz_trans(Vt, v_off[0][db][0], v_off[0][db][1]);
#pragma unroll
            for (int c4 = 0; c4 < 4; ++c4) {
                if (c4 + 1 < 4) {
#pragma unroll
                    for (int db = 0; db < D / 32; ++db) fv[(c4 + 1) & 1][db] = swz_trans(Vt, v_off[c4 + 1][db][0], v_off[c4 + 1][db][1]);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int db = 0; db < D / 32; ++db)
#pragma unroll
                    for (int b = 0; b < QB; ++b) oacc[b][db] = mfma16(fv[c4 & 1][db], pf[b][c4], oacc[b][db]);
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
#pragma unroll
            for (int c4 = 0; c4 < 4; ++c4)
#pragma unroll
                for (int db = 0; db < D / 32; ++db) {
                    const f16x8 a = swz_trans(Vt, v_off[c4][db][0], v_off[c4][db][1]);
#pragma unroll
                    for (int b = 0; b < QB; ++b) oacc[b][db] = mfma16(a, pf[b][c4], oacc[b][db]);
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

#pragma unroll
    for (int b = 0; b < QB; ++b) {
        const float ltot = half_sum(lsum[b]);
        const float inv = ltot > 0.f ? 1.f / ltot : 0.f;
        if (qvalid[b]) {
            const size_t row = (seg + qpos[b]) * D + 4 * h;
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const float x0 = oacc[b][db][4 * g + 0] * inv, x1 = oacc[b][db][4 * g + 1] * inv;
                    const float x2 = oacc[b][db][4 * g + 2] * inv, x3 = oacc[b][db][4 * g + 3] * inv;
                    const __bf16 y0 = (__bf16)x0, y1 = (__bf16)x1, y2 = (__bf16)x2, y3 = (__bf16)x3;
                    uint2 pk;
                    pk.x = (uint32_t)__builtin_bit_cast(uint16_t, y0) | ((uint32_t)__builtin_bit_cast(uint16_t, y1) << 16);
                    pk.y = (uint32_t)__builtin_bit_cast(uint16_t, y2) | ((uint32_t)__builtin_bit_cast(uint16_t, y3) << 16);
                    *reinterpret_cast<uint2*>(o + row + db * 32 + 8 * g) = pk;
                    if (o_f16) {   // the same values with 11 significant bits, for the backward's D = <dO, O>
                        const _Float16 z0 = (_Float16)x0, z1 = (_Float16)x1, z2 = (_Float16)x2, z3 = (_Float16)x3;
                        uint2 hk;
                        hk.x = (uint32_t)__builtin_bit_cast(uint16_t, z0) | ((uint32_t)__builtin_bit_cast(uint16_t, z1) << 16);
                        hk.y = (uint32_t)__builtin_bit_cast(uint16_t, z2) | ((uint32_t)__builtin_bit_cast(uint16_t, z3) << 16);
                        *reinterpret_cast<uint2*>(o_f16 + row + db * 32 + 8 * g) = hk;
                    }
                }
            if (h == 0) lse[seg + qpos[b]] = ltot > 0.f ? (m[b] * cexp + log2f(ltot)) * LN2 : -INFINITY;
        }
    }
}

template <int D, int NW, int QB>
static int launch_fwd_t(const void* q, const void* k, const void* v, const uint32_t* q_key, const uint32_t* k_key,
                        const int32_t* work, int n_work, int S, int T, float tau, int strict, void* o,
                        float* lse, void* o_f16, const int32_t* n_keep_q, hipStream_t st)
{
    constexpr size_t smem = (size_t)FwdRing<D>::NBUF * FwdRing<D>::BUF_BYTES;
    static std::atomic<unsigned long long> lds_allowed{0};
    { const int rc_ = allow_dynamic_lds(reinterpret_cast<const void*>(&attn_fwd_f16_kernel<D, NW, QB>), (int)smem, lds_allowed); if (rc_ != SCFA_OK) return rc_; }
    dim3 grid((unsigned)((size_t)S * n_work));
    hipLaunchKernelGGL((attn_fwd_f16_kernel<D, NW, QB>), grid, dim3(NW * 64), smem, st, (const uint16_t*)q,
                       (const uint16_t*)k, (const uint16_t*)v, q_key, k_key, work, n_work, S, T, tau,
                       strict, (uint16_t*)o, lse, (uint16_t*)o_f16, n_keep_q);
    SCFA_HIP_TRY(hipGetLastError());
    return SCFA_OK;
}

// workgroups of the forward kernel one CU holds at once (registers, LDS ring)
int occupancy_attn_fwd_bf16(int d, int* out)
{
    if (d == 64) {
        constexpr size_t smem = (size_t)FwdRing<64>::NBUF * FwdRing<64>::BUF_BYTES;
        SCFA_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_fwd_f16_kernel<64, 4, 1>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
        SCFA_HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(out, reinterpret_cast<const void*>(&attn_fwd_f16_kernel<64, 4, 1>), 256, smem));
        return SCFA_OK;
    }
    if (d == 128) {
        constexpr size_t smem = (size_t)FwdRing<128>::NBUF * FwdRing<128>::BUF_BYTES;
        SCFA_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_fwd_f16_kernel<128, 4, 1>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
        SCFA_HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(out, reinterpret_cast<const void*>(&attn_fwd_f16_kernel<128, 4, 1>), 256, smem));
        return SCFA_OK;
    }
    return SCFA_EUNSUPPORTED;
}

int launch_attn_fwd_bf16(const void* q, const void* k, const void* v, const uint32_t* q_key,
                         const uint32_t* k_key, const int32_t* work, int n_work, int S, int T, int d,
                         float tau, int strict, void* o, float* lse, void* o_f16, const int32_t* n_keep_q, hipStream_t st)
{
    ProfScope prof(SCFA_K_FWD, st);
    if (d == 64) return launch_fwd_t<64, 4, 1>(q, k, v, q_key, k_key, work, n_work, S, T, tau, strict, o, lse, o_f16, n_keep_q, st);
    if (d == 128) return launch_fwd_t<128, 4, 1>(q, k, v, q_key, k_key, work, n_work, S, T, tau, strict, o, lse, o_f16, n_keep_q, st);
    return SCFA_EUNSUPPORTED;
}

}  // namespace scfa
