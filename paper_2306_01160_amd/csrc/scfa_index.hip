// Integer / data-movement passes: stable sort by bucket, compaction of kept tokens,
// row gather, zero-fill of dropped rows.  All bit-exact; HBM- or latency-bound.
//
// Sort (paper Sec. 3.2) and compaction (Sec. 3.1) are the same operation: a stable
// counting sort of the positions 0..T-1 by a small key (bucket id, or "dropped" flag).
// One workgroup of 16 wavefronts owns one (batch, head) segment: every wavefront
// histograms a contiguous run of the sequence, the per-(key, wavefront) counts are
// turned into start offsets in (key, wavefront) order, and every wavefront then ranks
// its run 64 tokens at a time with wave-wide ballots -- tokens keep their relative
// order inside a key, which is what makes the sort stable.
#include "scfa_common.hpp"

namespace scfa {

constexpr int SORT_WAVES = 16;
constexpr int SORT_THREADS = SORT_WAVES * 64;

template <bool KEEP_MODE>
__device__ __forceinline__ int load_key(const void* keys, size_t i, int nb)
{
    if (KEEP_MODE) {
        return reinterpret_cast<const uint8_t*>(keys)[i] != 0 ? 0 : 1;
    } else {
        int k = reinterpret_cast<const int32_t*>(keys)[i];
        k = k < 0 ? 0 : k;
        return k >= nb ? nb - 1 : k;
    }
}

// keys: [S,T] int32 bucket ids, or uint8 keep flags in KEEP_MODE (key 0 = kept, 1 = dropped).
// off_out: [S,nb+1] in bucket mode; [S] kept count in KEEP_MODE.
// One launch sorts up to two independent key tensors (queries and keys of the same shape):
// workgroups [0, S) take problem 0, workgroups [S, 2S) problem 1.
struct SortProblem {
    const void* keys;
    int32_t* idx_out;
    int32_t* key_sorted_out;
    int32_t* off_out;
    uint32_t* sort_key_out;   // bucket << 24 | position of every sorted row (nullable)
};

constexpr int SORT_PREFETCH = 16;  // 64-token steps whose keys are loaded together

// Long sequences in few segments leave most of the chip idle with one workgroup per segment, so a
// segment can be cut into n_chunks runs of chunk_len tokens (a multiple of 64 * SORT_WAVES), one
// workgroup each: a first kernel counts the keys of every chunk, the sort kernel then starts each
// key of its chunk after all smaller keys of the segment and after the same key in earlier chunks.
// Up to SELF_COUNT_MAX_T tokens per segment the first kernel is not launched: every workgroup of the
// sort kernel counts the keys of the other chunks itself (at most 16 more keys per thread, read from
// L2), which costs less than a launch.
constexpr int COUNT_THREADS = 256;
constexpr int SELF_COUNT_MAX_T = 16384;

template <bool KEEP_MODE>
__global__ __launch_bounds__(COUNT_THREADS) void sort_chunk_count_kernel(
    const void* keys0, const void* keys1, int S, int T, int nb, int n_chunks, int chunk_len,
    int32_t* __restrict__ chunk_counts /* [problem][S][n_chunks][nb] */)
{
    extern __shared__ int32_t smem[];
    const int c = blockIdx.x % n_chunks;
    const int ps = blockIdx.x / n_chunks;       // problem * S + segment
    const void* __restrict__ keys = ps >= S ? keys1 : keys0;
    const size_t seg = (size_t)(ps >= S ? ps - S : ps) * T;
    for (int k = threadIdx.x; k < nb; k += COUNT_THREADS) smem[k] = 0;
    __syncthreads();
    const int t0 = c * chunk_len, t1 = min(T, t0 + chunk_len);
    for (int t = t0 + threadIdx.x; t < t1; t += COUNT_THREADS) atomicAdd(&smem[load_key<KEEP_MODE>(keys, seg + t, nb)], 1);
    __syncthreads();
    for (int k = threadIdx.x; k < nb; k += COUNT_THREADS) chunk_counts[((size_t)ps * n_chunks + c) * nb + k] = smem[k];
}

template <bool KEEP_MODE>
__global__ __launch_bounds__(SORT_THREADS) void stable_sort_small_keys_kernel(
    SortProblem p0, SortProblem p1, int S, int T, int nb, int nbits, int n_chunks, int chunk_len,
    const int32_t* __restrict__ chunk_counts)
{
    extern __shared__ int32_t smem[];
    int32_t* hist = smem;                       // [SORT_WAVES][nb]  counts, then running bases
    int32_t* tot = smem + SORT_WAVES * nb;      // [nb+1]
    int32_t* before = tot + nb + 1;             // [nb] tokens of the key in earlier chunks of the segment
    int32_t* later = before + nb;               // [nb] ... in later chunks (only when this kernel counts them itself)
    const bool self_count = n_chunks > 1 && chunk_counts == nullptr;
    const int chunk = blockIdx.x % n_chunks;
    const int ps = blockIdx.x / n_chunks;
    const bool second = ps >= S;
    const int s = second ? ps - S : ps;
    const void* __restrict__ keys = second ? p1.keys : p0.keys;
    int32_t* __restrict__ idx_out = second ? p1.idx_out : p0.idx_out;
    int32_t* __restrict__ key_sorted_out = second ? p1.key_sorted_out : p0.key_sorted_out;
    int32_t* __restrict__ off_out = second ? p1.off_out : p0.off_out;
    uint32_t* __restrict__ sort_key_out = second ? p1.sort_key_out : p0.sort_key_out;
    const int wave = threadIdx.x >> 6;
    const int lane = threadIdx.x & 63;
    const size_t seg = (size_t)s * T;

    // contiguous run of this wavefront inside the workgroup's chunk, a multiple of 64 tokens
    const int c0 = chunk * chunk_len, c1 = min(T, c0 + chunk_len);
    int run = (c1 - c0 + SORT_WAVES - 1) / SORT_WAVES;
    run = (run + 63) & ~63;
    const int r0 = min(c0 + wave * run, c1);
    const int r1 = min(r0 + run, c1);

    for (int i = threadIdx.x; i < SORT_WAVES * nb; i += SORT_THREADS) hist[i] = 0;
    if (self_count)
        for (int i = threadIdx.x; i < nb; i += SORT_THREADS) { before[i] = 0; later[i] = 0; }
    __syncthreads();
    if (self_count) {   // the other chunks of the segment: [0, c0) and [c1, T), eight keys per thread in flight
        const int n_other = c0 + (T - c1);
        for (int i0 = threadIdx.x; i0 < n_other; i0 += 8 * SORT_THREADS) {
            int kv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = i0 + u * SORT_THREADS;
                kv[u] = i < n_other ? load_key<KEEP_MODE>(keys, seg + (i < c0 ? i : i - c0 + c1), nb) : -1;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (kv[u] >= 0) atomicAdd(i0 + u * SORT_THREADS < c0 ? &before[kv[u]] : &later[kv[u]], 1);
        }
    }
    // histogram of the run; the keys of SORT_PREFETCH 64-token steps are loaded together so
    // that the memory latency is paid once per group, not once per step.  A run of at most
    // one group (T <= 16 * 64 * SORT_PREFETCH) keeps its keys in registers for the ranking.
    const bool single_group = r1 - r0 <= 64 * SORT_PREFETCH;
    int keyv[SORT_PREFETCH];
    for (int g0 = r0; g0 < r1; g0 += 64 * SORT_PREFETCH) {
#pragma unroll
        for (int u = 0; u < SORT_PREFETCH; ++u) {
            const int t = g0 + 64 * u + lane;
            keyv[u] = t < r1 ? load_key<KEEP_MODE>(keys, seg + t, nb) : -1;
        }
#pragma unroll
        for (int u = 0; u < SORT_PREFETCH; ++u)
            if (keyv[u] >= 0) atomicAdd(&hist[wave * nb + keyv[u]], 1);
    }
    __syncthreads();

    // per key: exclusive prefix over wavefronts (in place) and the key total of the segment
    for (int k = threadIdx.x; k < nb; k += SORT_THREADS) {
        int acc = 0;
        for (int w = 0; w < SORT_WAVES; ++w) {
            const int c = hist[w * nb + k];
            hist[w * nb + k] = acc;
            acc += c;
        }
        int earlier = 0;
        if (self_count) {
            earlier = before[k];
            acc += earlier + later[k];
        } else if (n_chunks > 1) {   // the segment's total and the part of it that lies in earlier chunks
            const int32_t* cc = chunk_counts + (size_t)ps * n_chunks * nb + k;
            acc = 0;
            for (int c = 0; c < n_chunks; ++c) {
                if (c == chunk) earlier = acc;
                acc += cc[(size_t)c * nb];
            }
        }
        before[k] = earlier;
        tot[k] = acc;
    }
    __syncthreads();
    if (threadIdx.x == 0) {   // exclusive prefix over keys (nb <= 256)
        int acc = 0;
        for (int k = 0; k < nb; ++k) {
            const int c = tot[k];
            tot[k] = acc;
            acc += c;
        }
        tot[nb] = acc;
    }
    __syncthreads();
    if (chunk == 0) {
        if (KEEP_MODE) {
            if (threadIdx.x == 0) off_out[s] = tot[1];
        } else {
            for (int k = threadIdx.x; k <= nb; k += SORT_THREADS) off_out[(size_t)s * (nb + 1) + k] = tot[k];
        }
    }
    for (int i = threadIdx.x; i < SORT_WAVES * nb; i += SORT_THREADS) hist[i] += tot[i % nb] + before[i % nb];
    __syncthreads();

    // rank and scatter, 64 consecutive tokens per step, keys again loaded a group at a time
    int32_t* base = hist + wave * nb;
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    for (int g0 = r0; g0 < r1; g0 += 64 * SORT_PREFETCH) {
        if (!single_group) {
#pragma unroll
            for (int u = 0; u < SORT_PREFETCH; ++u) {
                const int t = g0 + 64 * u + lane;
                keyv[u] = t < r1 ? load_key<KEEP_MODE>(keys, seg + t, nb) : -1;
            }
        }
#pragma unroll
        for (int u = 0; u < SORT_PREFETCH; ++u) {
            const int t = g0 + 64 * u + lane;
            if (g0 + 64 * u >= r1) break;       // wave-uniform
            const bool valid = t < r1;
            const int key = valid ? keyv[u] : 0;
            unsigned long long same = __ballot(valid);
            for (int b = 0; b < nbits; ++b) {
                const bool bit = (key >> b) & 1;
                const unsigned long long m = __ballot(bit);
                same &= bit ? m : ~m;
            }
            const int rank = __popcll(same & lt_mask);
            const int cnt = __popcll(same);
            int pos = 0;
            if (valid) pos = base[key] + rank;
            __builtin_amdgcn_wave_barrier();
            if (valid && rank == 0) base[key] += cnt;
            __builtin_amdgcn_wave_barrier();
            if (valid) {
                idx_out[seg + pos] = t;
                if (key_sorted_out) key_sorted_out[seg + pos] = key;
                if (sort_key_out) sort_key_out[seg + pos] = ((uint32_t)key << KEY_POS_BITS) | (uint32_t)t;
            }
        }
    }
}

// n_problems: 1 or 2 (bucket1 etc. ignored for 1)
// Chunks per segment for n_wg = segments x problems workgroups: enough to fill the chip once, but
// chunks of at least 4096 tokens; 1 for short sequences.  Host arithmetic; the workspace query and
// the launchers must agree.
int sort_chunks(int n_wg, int T)
{
    if (T < 8192) return 1;
    int c = (256 + n_wg - 1) / n_wg;
    if (c > T / 4096) c = T / 4096;
    if (c > 64) c = 64;
    return c < 1 ? 1 : c;
}

static int sort_chunk_len(int T, int n_chunks)
{
    const int unit = 64 * SORT_WAVES;
    return ((T + n_chunks - 1) / n_chunks + unit - 1) / unit * unit;
}

size_t sort_workspace_bytes(int n_problems, int S, int T, int nb)
{
    const int c = sort_chunks(S * n_problems, T);
    return c > 1 ? sizeof(int32_t) * (size_t)n_problems * S * c * nb : 0;
}

template <bool KEEP_MODE>
static int launch_sort_t(int kid, int n_problems, const SortProblem& p0, const SortProblem& p1, int S, int T, int nb,
                         int nbits, void* ws, size_t ws_bytes, hipStream_t st, bool timed = true,
                         bool self_count_ok = true)
{
    const size_t smem = sizeof(int32_t) * ((size_t)SORT_WAVES * nb + 3 * (size_t)nb + 1);
    int n_chunks = sort_chunks(S * n_problems, T);
    const bool self_count = self_count_ok && T <= SELF_COUNT_MAX_T;   // the sort kernel counts the other chunks itself
    if (!self_count && (!ws || ws_bytes < sort_workspace_bytes(n_problems, S, T, nb))) n_chunks = 1;   // no scratch: one workgroup per segment
    int chunk_len = sort_chunk_len(T, n_chunks);
    n_chunks = (T + chunk_len - 1) / chunk_len;      // rounding the length up may leave fewer chunks
    ProfScope prof(timed ? kid : -1, st);            // the timers create events: not on the allocation-free path
    if (n_chunks > 1 && !self_count)
        hipLaunchKernelGGL(sort_chunk_count_kernel<KEEP_MODE>, dim3(S * n_problems * n_chunks), dim3(COUNT_THREADS),
                           sizeof(int32_t) * nb, st, p0.keys, p1.keys, S, T, nb, n_chunks, chunk_len, (int32_t*)ws);
    hipLaunchKernelGGL(stable_sort_small_keys_kernel<KEEP_MODE>, dim3(S * n_problems * n_chunks), dim3(SORT_THREADS), smem,
                       st, p0, p1, S, T, nb, nbits, n_chunks, chunk_len, self_count ? nullptr : (const int32_t*)ws);
    SCFA_HIP_TRY(hipGetLastError());
    return SCFA_OK;
}

int launch_sort_by_bucket(int n_problems, const int32_t* bucket0, const int32_t* bucket1, int S, int T, int nb,
                          int32_t* idx0, int32_t* sorted0, int32_t* off0, uint32_t* key0, int32_t* idx1,
                          int32_t* sorted1, int32_t* off1, uint32_t* key1, void* ws, size_t ws_bytes, hipStream_t st)
{
    int nbits = 0;
    while ((1 << nbits) < nb) ++nbits;
    const SortProblem p0{bucket0, idx0, sorted0, off0, key0}, p1{bucket1, idx1, sorted1, off1, key1};
    return launch_sort_t<false>(SCFA_K_SORT, n_problems, p0, p1, S, T, nb, nbits, ws, ws_bytes, st);
}

// ---------------------------------------------------------------------------
// The sort with the chunk counters in memory the library owns: a file-scope device array instead
// of a caller workspace, for callers that cannot allocate.  Every device holds its own copy of the
// array at its own address; the address is looked up once per device (with that device current)
// and kept.  In host code the array's name is only a handle for that lookup, never an address.
static __device__ __align__(256) unsigned char scratch[SCFA_STATIC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
static std::atomic<void*> g_scratch_ptr[MAX_DEVICES];

// device address of `scratch` on the device `st` belongs to, which must be the current device
static int static_scratch(hipStream_t st, void** out)
{
    int dev = 0;
    SCFA_HIP_TRY(hipGetDevice(&dev));
    if (st) {
        int sdev = -1;
        SCFA_HIP_TRY(hipStreamGetDevice(st, &sdev));
        if (sdev != dev) return SCFA_EINVAL;
    }
    if (dev < 0 || dev >= MAX_DEVICES) return SCFA_EUNSUPPORTED;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        SCFA_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return SCFA_EHIP;
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return SCFA_OK;
}

int launch_sort_by_bucket_static(const int32_t* bucket, int S, int T, int nb, int32_t* idx, int32_t* sorted,
                                 int32_t* off, uint32_t* key, hipStream_t st)
{
    // the chunk counters must fit the array: nothing is launched otherwise
    const size_t need = sort_workspace_bytes(1, S, T, nb);
    if (need > SCFA_STATIC_SCRATCH_BYTES) return SCFA_EWORKSPACE;
    void* ptr = nullptr;
    const int rc = static_scratch(st, &ptr);
    if (rc != SCFA_OK) return rc;
    int nbits = 0;
    while ((1 << nbits) < nb) ++nbits;
    const SortProblem p0{bucket, idx, sorted, off, key}, p1{nullptr, nullptr, nullptr, nullptr, nullptr};
    // every counter the sort kernel reads is written by the counting kernel of the same call, so
    // what an earlier call left in the array does not matter
    return launch_sort_t<false>(SCFA_K_SORT, 1, p0, p1, S, T, nb, nbits, ptr, SCFA_STATIC_SCRATCH_BYTES, st, false, false);
}

int launch_compact_keep(int n_problems, const uint8_t* keep0, const uint8_t* keep1, int S, int T, int32_t* idx0,
                        int32_t* count0, int32_t* idx1, int32_t* count1, void* ws, size_t ws_bytes, hipStream_t st)
{
    const SortProblem p0{keep0, idx0, nullptr, count0, nullptr}, p1{keep1, idx1, nullptr, count1, nullptr};
    return launch_sort_t<true>(SCFA_K_COMPACT, n_problems, p0, p1, S, T, 2, 1, ws, ws_bytes, st);
}

// ---------------------------------------------------------------------------
// Row gather: 16 bytes per thread, a row of d elements is row_bytes/16 consecutive
// lanes, so every row is read and written as whole cache lines.  One launch serves up to
// three tensors of the same shape (blockIdx.z): Q, K and V of one attention call.
struct GatherProblem {
    const void* x;
    const int32_t* idx;
    const int32_t* count;
    void* out;
    float scale;
};
struct GatherBatch { GatherProblem p[3]; };

// MODE 0: bit-exact copy; 1: bf16 -> fp16 (times scale, one rounding to nearest even; with
// scale 1 exact for magnitudes in [2^-17, 65504], larger ones become infinite and NaN stays
// NaN, so that an input outside the compute format shows in the results instead of being
// replaced by a finite value); 2: fp32 times scale (one rounding)
template <int MODE>
__global__ __launch_bounds__(256) void gather_rows_kernel(GatherBatch batch, int T, int chunks_per_row)
{
    const GatherProblem& pr = batch.p[blockIdx.z];
    const int s = blockIdx.y;
    const int n = pr.count ? pr.count[s] : T;
    const long long g = (long long)blockIdx.x * 256 + threadIdx.x;
    const int r = (int)(g / chunks_per_row);
    const int c = (int)(g % chunks_per_row);
    if (r >= n) return;
    const int src = pr.idx[(size_t)s * T + r];
    const uint4 v = reinterpret_cast<const uint4*>(pr.x)[((size_t)s * T + src) * chunks_per_row + c];
    uint4 res = v;
    if (MODE == 1) {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
        uint32_t o[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float lo = __uint_as_float(w[i] << 16) * pr.scale, hi = __uint_as_float(w[i] & 0xffff0000u) * pr.scale;
            const _Float16 a = (_Float16)lo, b = (_Float16)hi;   // IEEE conversion: beyond the fp16 range -> inf, NaN stays NaN
            o[i] = (uint32_t)__builtin_bit_cast(uint16_t, a) | ((uint32_t)__builtin_bit_cast(uint16_t, b) << 16);
        }
        res = make_uint4(o[0], o[1], o[2], o[3]);
    } else if (MODE == 2) {
        res = make_uint4(__float_as_uint(__uint_as_float(v.x) * pr.scale), __float_as_uint(__uint_as_float(v.y) * pr.scale),
                         __float_as_uint(__uint_as_float(v.z) * pr.scale), __float_as_uint(__uint_as_float(v.w) * pr.scale));
    }
    reinterpret_cast<uint4*>(pr.out)[((size_t)s * T + r) * chunks_per_row + c] = res;
}

// mode as in the kernel; n_tensors 1..3 problems of identical shape
int launch_gather_rows(int n_tensors, const void* const* x, const int32_t* const* idx, const int32_t* const* count,
                       const float* scale, void* const* out, int S, int T, int row_bytes, int mode, hipStream_t st)
{
    GatherBatch batch{};
    for (int i = 0; i < n_tensors; ++i) batch.p[i] = GatherProblem{x[i], idx[i], count[i], out[i], scale[i]};
    const int cpr = row_bytes / 16;
    const long long total = (long long)T * cpr;
    dim3 grid((unsigned)((total + 255) / 256), S, n_tensors);
    ProfScope prof(SCFA_K_GATHER, st);
    if (mode == 0)
        hipLaunchKernelGGL(gather_rows_kernel<0>, grid, dim3(256), 0, st, batch, T, cpr);
    else if (mode == 1)
        hipLaunchKernelGGL(gather_rows_kernel<1>, grid, dim3(256), 0, st, batch, T, cpr);
    else
        hipLaunchKernelGGL(gather_rows_kernel<2>, grid, dim3(256), 0, st, batch, T, cpr);
    SCFA_HIP_TRY(hipGetLastError());
    return SCFA_OK;
}

// ---------------------------------------------------------------------------
// Bucket ids outside [0, nb): counted, one atomic per wavefront that found any.  The first
// kernel clears the counter (no memset node: the pair may be captured in a graph).
__global__ void clear_counter_kernel(int32_t* __restrict__ counter) { *counter = 0; }

__global__ __launch_bounds__(256) void count_invalid_buckets_kernel(const int32_t* __restrict__ bucket, long long n,
                                                                    int nb, int32_t* __restrict__ counter)
{
    int bad = 0;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long long)gridDim.x * 256) {
        const int b = bucket[i];
        bad += (b < 0 || b >= nb) ? 1 : 0;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) bad += __shfl_xor(bad, off);
    if ((threadIdx.x & 63) == 0 && bad > 0) atomicAdd(counter, bad);
}

int launch_count_invalid_buckets(const int32_t* bucket, long long n, int nb, int32_t* counter, hipStream_t st)
{
    hipLaunchKernelGGL(clear_counter_kernel, dim3(1), dim3(1), 0, st, counter);
    SCFA_HIP_TRY(hipGetLastError());
    if (n > 0) {
        const long long blocks = (n + 256 * 8 - 1) / (256 * 8);
        hipLaunchKernelGGL(count_invalid_buckets_kernel, dim3((unsigned)(blocks < 4096 ? blocks : 4096)), dim3(256), 0, st,
                           bucket, n, nb, counter);
        SCFA_HIP_TRY(hipGetLastError());
    }
    return SCFA_OK;
}

// ---------------------------------------------------------------------------
// Zero the rows idx[s, count[s] .. T) of up to two [S,T,row] outputs (original order)
// and set vec[s, idx] = vec_value: the dropped queries / keys of QK-dropping.
__global__ __launch_bounds__(256) void zero_rows_kernel(const int32_t* __restrict__ idx,
                                                        const int32_t* __restrict__ count, int T,
                                                        int chunks_per_row, uint4* __restrict__ out0,
                                                        uint4* __restrict__ out1,
                                                        float* __restrict__ vec, float vec_value)
{
    const int s = blockIdx.y;
    const int n = count[s];
    const long long g = (long long)blockIdx.x * 256 + threadIdx.x;
    const int r = n + (int)(g / chunks_per_row);
    const int c = (int)(g % chunks_per_row);
    if (r >= T) return;
    const int dst = idx[(size_t)s * T + r];
    const uint4 z = make_uint4(0u, 0u, 0u, 0u);
    const size_t o = ((size_t)s * T + dst) * chunks_per_row + c;
    if (out0) out0[o] = z;
    if (out1) out1[o] = z;
    if (vec && c == 0) vec[(size_t)s * T + dst] = vec_value;
}

int launch_zero_rows(const int32_t* idx, const int32_t* count, int S, int T, int row_bytes,
                     void* out0, void* out1, float* vec, float vec_value, hipStream_t st)
{
    const int cpr = row_bytes / 16;
    const long long total = (long long)T * cpr;
    dim3 grid((unsigned)((total + 255) / 256), S);
    ProfScope prof(SCFA_K_FILL, st);
    hipLaunchKernelGGL(zero_rows_kernel, grid, dim3(256), 0, st, idx, count, T, cpr, (uint4*)out0,
                       (uint4*)out1, vec, vec_value);
    SCFA_HIP_TRY(hipGetLastError());
    return SCFA_OK;
}

}  // namespace scfa
