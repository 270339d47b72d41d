// LSH bucketing in front of the hash-sparse path (paper Sec. 4.2 "Hashing mechanism": the
// cross-polytope scheme of Andoni et al. with a chosen number of hash codes).  For every
// row x of a [S,T,d] tensor and the projection R of its head (d x r, r = nb / 2):
//     bucket = argmax over [x R, -x R]        (lowest index on ties)
// Two kernels.  bf16 rows with at most 32 projection columns go to the matrix cores (second half of this file).  The
// vector-unit kernel below serves fp32 rows and wider projections: x is read once (16 bytes per lane, a row is d/8 adjacent
// lanes), R sits in LDS, 4 bytes are written per row.  Its r dot products are formed eight columns at a time: each
// lane multiplies its 8 elements into partial sums (its 8 x 8 block of R in registers, reused
// for eight rows), the row's lanes add them up with cross-lane shuffles, and a running
// (value, index) maximum over +-p is kept.  Arithmetic is
// fp32 (fused multiply-adds in element order inside a lane, then a pairwise tree over lanes).
#include "scfa_common.hpp"
#include "scfa_mma.hpp"

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

// ---- bf16 rows, at most 32 projection columns: the contraction on the matrix cores -------------------------------------------
// P^T = R^T x^T with v_mfma_f32_32x32x16_bf16: the M side is the projection column (zero past r), the N side the row, so a lane ends
// up with 16 of the 32 projections of ITS row (the other half-lane holds the other 16) and the argmax is 16 compares in a lane plus
// one exchange.  The rows are bf16 already and go into the B operand as they are, 16 bytes per lane straight from global memory
// (lane = row, eight consecutive elements); R is fp32 and is split into three bf16 pieces whose sum is R to 24 bits, so that
// every product is exact in fp32 and the result differs from an fp32 dot product only by the order of its sums.  With the vector
// units this kernel was bound by their arithmetic as r grew (3.2 TB/s at nb = 8, 0.67 TB/s at nb = 64 on d = 64 rows).
using bf16x8 = __bf16 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ uint32_t bf16_rne_bits(float x)   // finite x
{
    const uint32_t u = __float_as_uint(x);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

template <int D>
__global__ __launch_bounds__(256) void lsh_buckets_mfma_kernel(LshProblem p0, LshProblem p1, const float* __restrict__ R,
                                                               int H, int T, int r, int tiles_per_wave)
{
    constexpr int KS = D / 16;            // contraction steps of 16
    constexpr int CH = D / 8;             // 16-byte chunks per row
    constexpr int ROUNDS = 32 * CH / 64;  // loads of a wavefront per 32-row tile (1 KiB each)
    constexpr int TILE_BYTES = 32 * D * 2;
    extern __shared__ __attribute__((aligned(256))) unsigned char lsh_smem[];   // [4 wavefronts][2 buffers][32 rows x D bf16], swizzled
    const int s = blockIdx.y;
    const LshProblem& pr = blockIdx.z ? p1 : p0;
    const float* Rh = R + (size_t)(s % H) * D * r;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6), l32 = lane & 31, h = lane >> 5;

    // Rows travel global memory -> LDS asynchronously, a kilobyte (8 or 4 whole rows) per instruction, each wavefront its own 32
    // rows into its own two buffers (no workgroup barrier anywhere); the chunk a lane fetches is chosen so that the tile lands swizzled.
    const int first_tile = (blockIdx.x * 4 + wave) * tiles_per_wave;    // 32-row tiles of this wavefront: first_tile ...
    const u32x4 desc = make_desc(reinterpret_cast<const uint16_t*>(pr.x) + (size_t)s * T * D, (uint32_t)((size_t)T * D * 2));
    const uint32_t lds_wave = lds_address(lsh_smem) + (uint32_t)(wave * 2 * TILE_BYTES);
    int voff[ROUNDS];
#pragma unroll
    for (int u = 0; u < ROUNDS; ++u) {
        const int pos = u * 64 + lane, row = pos / CH, slot = pos % CH;
        voff[u] = (row * CH + (slot ^ swz<D>(row))) * 16;
    }
    auto issue = [&](int t, int buf) {    // tile t of this wavefront; rows past T land as zeros
#pragma unroll
        for (int u = 0; u < ROUNDS; ++u)
            async_load16(desc, lds_wave + (uint32_t)(buf * TILE_BYTES + u * 1024), voff[u], (first_tile + t) * TILE_BYTES);
    };
    issue(0, 0);
    if (tiles_per_wave > 1) issue(1, 1);

    // A operand: column l32 of R, rows 16 kk + 8 h + 0..7, as three bf16 pieces (formed while the first rows travel)
    bf16x8 a1[KS], a2[KS], a3[KS];
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
        uint32_t w1[4], w2[4], w3[4];
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
            uint32_t b1[2], b2[2], b3[2];
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const float v = l32 < r ? Rh[(size_t)(kk * 16 + h * 8 + 2 * e2 + q) * r + l32] : 0.f;
                b1[q] = bf16_rne_bits(v);
                const float rem1 = v - __uint_as_float(b1[q] << 16);
                b2[q] = bf16_rne_bits(rem1);
                const float rem2 = rem1 - __uint_as_float(b2[q] << 16);
                b3[q] = bf16_rne_bits(rem2);
            }
            w1[e2] = b1[0] | (b1[1] << 16); w2[e2] = b2[0] | (b2[1] << 16); w3[e2] = b3[0] | (b3[1] << 16);
        }
        a1[kk] = __builtin_bit_cast(bf16x8, make_uint4(w1[0], w1[1], w1[2], w1[3]));
        a2[kk] = __builtin_bit_cast(bf16x8, make_uint4(w2[0], w2[1], w2[2], w2[3]));
        a3[kk] = __builtin_bit_cast(bf16x8, make_uint4(w3[0], w3[1], w3[2], w3[3]));
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // R's loads are the compiler's; from here on only tile loads are in flight

    for (int t = 0; t < tiles_per_wave; ++t) {
        const int buf = t & 1;
        if (t + 1 < tiles_per_wave) wait_async<ROUNDS>(); else wait_async<0>();
        const uint16_t* tile = reinterpret_cast<const uint16_t*>(lsh_smem + (size_t)(wave * 2 + buf) * TILE_BYTES);
        bf16x8 b[KS];
#pragma unroll
        for (int kk = 0; kk < KS; ++kk)
            b[kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(tile + swz_offset<D>(l32, kk * 16 + h * 8)));
        f32x16 acc = zero16();
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) {      // smallest pieces first
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a3[kk], b[kk], acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a2[kk], b[kk], acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1[kk], b[kk], acc, 0, 0, 0);
        }
        // the fragments are in registers (the matrix instructions above have read them): the buffer may be refilled
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        if (t + 2 < tiles_per_wave) issue(t + 2, buf);
        // register i of the lane: projection column 8 (i / 4) + 4 h + i % 4 of its row.  Candidates in index order are
        // +p_0 .. +p_{r-1}, -p_0 .. -p_{r-1} and the first maximum wins: a strictly larger value replaces the choice inside each
        // half (columns ascend with i), a tie between lanes goes to the lower index, a tie between halves to the positive one.
        float bp = -INFINITY, bn = -INFINITY;
        int ip = 0, in_ = r;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int c = 8 * (i >> 2) + 4 * h + (i & 3);
            const float pv = c < r ? acc[i] : -INFINITY, nv = c < r ? -acc[i] : -INFINITY;
            if (pv > bp) { bp = pv; ip = c; }
            if (nv > bn) { bn = nv; in_ = r + c; }
        }
        const float obp = __shfl_xor(bp, 32), obn = __shfl_xor(bn, 32);
        const int oip = __shfl_xor(ip, 32), oin = __shfl_xor(in_, 32);
        if (obp > bp || (obp == bp && oip < ip)) { bp = obp; ip = oip; }
        if (obn > bn || (obn == bn && oin < in_)) { bn = obn; in_ = oin; }
        const int row = (first_tile + t) * 32 + l32;
        if (h == 0 && row < T) pr.bucket_out[(size_t)s * T + row] = bn > bp ? in_ : ip;
    }
}

int launch_lsh_buckets(int n_problems, const void* x0, const void* x1, const float* R, int S, int H, int T, int d,
                       int nb, bool bf16, int32_t* out0, int32_t* out1, hipStream_t st)
{
    const int r = nb / 2;
    const size_t smem = sizeof(float) * (size_t)d * r;
    const LshProblem p0{x0, out0}, p1{x1, out1};
    if (bf16 && r <= 32 && (d == 64 || d == 128) && (size_t)T * d * 2 < 0x7f000000ull) {   // the contraction on the matrix cores (byte offsets into a segment are 32-bit)
        ProfScope prof(SCFA_K_LSH, st);
        // a wavefront takes tiles_per_wave consecutive 32-row tiles: about three workgroups per CU in all (every workgroup first
        // forms its copy of R's pieces; measured at d = 64, 393216 rows x 2: 29 / 26 / 23 / 25 / 38 us with 3 / 4 / 8 / 16 / 32 tiles)
        const int n_tiles = (T + 31) / 32;
        int tpw = (int)(((long long)n_tiles * S * n_problems + 4 * 768 - 1) / (4 * 768));
        tpw = tpw < 2 ? 2 : tpw > 64 ? 64 : tpw;
        dim3 grid((unsigned)((n_tiles + 4 * tpw - 1) / (4 * tpw)), S, n_problems);
        const size_t smem = (size_t)4 * 2 * 32 * d * 2;
        static std::atomic<unsigned long long> lds_allowed_64{0}, lds_allowed_128{0};
        if (d == 64) {
            const int rc_ = allow_dynamic_lds(reinterpret_cast<const void*>(&lsh_buckets_mfma_kernel<64>), (int)smem, lds_allowed_64);
            if (rc_ != SCFA_OK) return rc_;
            hipLaunchKernelGGL((lsh_buckets_mfma_kernel<64>), grid, dim3(256), smem, st, p0, p1, R, H, T, r, tpw);
        } else {
            const int rc_ = allow_dynamic_lds(reinterpret_cast<const void*>(&lsh_buckets_mfma_kernel<128>), (int)smem, lds_allowed_128);
            if (rc_ != SCFA_OK) return rc_;
            hipLaunchKernelGGL((lsh_buckets_mfma_kernel<128>), grid, dim3(256), smem, st, p0, p1, R, H, T, r, tpw);
        }
        SCFA_HIP_TRY(hipGetLastError());
        return SCFA_OK;
    }
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
