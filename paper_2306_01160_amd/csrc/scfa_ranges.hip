// Tile-skip schedule (paper Sec. 3.1: j_stop from the key / query index vectors;
// Sec. 3.2: j_start, j_stop from the bucket ids, then the causal refinement).
//
// The paper's kernels scan blocks of the index vectors inside every program.  Here
// the schedule is a pass of its own, and because this library owns the tiling it
// anchors tiles at bucket boundaries: a work item is a tile of query rows of ONE
// bucket together with the range of keys of the same bucket that the causal test
// can let through.  Positions are increasing inside a bucket (stable sort), so both
// range ends are binary searches in the key (query) index vector:
//   forward item : keys with position <= largest query position of the tile
//                  (and the prefix with position <= smallest query position needs no mask)
//   backward item: queries with position >= smallest key position of the tile
//                  (only those with position < largest key position need a mask)
// Buckets with fewer rows than a tile would leave most of every tile empty, so consecutive small
// buckets are put together: as many whole buckets as fit one tile of the tiled side form one
// item that spans all their rows on both sides.  The kernels tell the buckets of such an item
// apart by the sort keys (bucket << 24 | position), which they test in every tile of it.
// Items of a segment are emitted bucket pair by bucket pair, and inside a pair in order of
// decreasing work.  Workgroups that run at the same time then share the keys / values
// (forward) or queries / dO rows (backward) of one or two buckets, which stay in the L2 of
// their XCD (measured at 8 buckets of 2048: 0.15-0.2 GB fetched from memory per attention
// kernel instead of 0.6 GB with a purely work-ordered list), while the last workgroups of a
// launch are still the short items.
//
// One workgroup builds one list of one segment (the forward and the backward list are
// independent).  The index vector that is searched is first copied into LDS when it fits,
// so the dependent steps of the binary searches cost LDS, not global-memory, latency; when it
// does not fit, every 2^shift-th entry is copied and a search ends with <= shift steps in global
// memory.
#include "scfa_common.hpp"

namespace scfa {

constexpr int RANGES_THREADS = 512;

// number of entries of a[0..n) that are <= v (a increasing)
__device__ __forceinline__ int count_le(const int32_t* __restrict__ a, int n, int v)
{
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (a[mid] <= v) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// number of entries of a[0..n) that are < v
__device__ __forceinline__ int count_lt(const int32_t* __restrict__ a, int n, int v)
{
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (a[mid] < v) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// The searched vector: `g` in global memory and lds[i] = g[i << shift] (shift 0: all of it).
struct Searched { const int32_t* g; const int32_t* lds; int shift; };

// number of entries of g[begin, begin + n) that are <= v (LE) or < v
template <bool LE>
__device__ __forceinline__ int count_in(const Searched& a, int begin, int n, int v)
{
    if (a.shift == 0) return LE ? count_le(a.lds + begin, n, v) : count_lt(a.lds + begin, n, v);
    int lo = begin, hi = begin + n;                        // the answer is a position in [lo, hi]
    const int j0 = (begin + (1 << a.shift) - 1) >> a.shift, j1 = (begin + n - 1) >> a.shift;   // samples inside
    if (n > 0 && j0 <= j1) {
        const int c = LE ? count_le(a.lds + j0, j1 - j0 + 1, v) : count_lt(a.lds + j0, j1 - j0 + 1, v);
        if (c > 0) lo = ((j0 + c - 1) << a.shift) + 1;     // that sample and all before it count
        if (c <= j1 - j0) hi = (j0 + c) << a.shift;        // the next sample does not
    }
    return lo - begin + (LE ? count_le(a.g + lo, hi - lo, v) : count_lt(a.g + lo, hi - lo, v));
}

constexpr int ORDER_GROUP = 2;   // buckets whose items are dispatched together

struct Item { int a_begin, a_count, b_begin, b_count, b_extra, bucket, n_buckets; };

// ascending sort key: bucket pair first, then decreasing length of the ranged side (< 2^24)
__device__ __forceinline__ int order_key(int bucket, int b_count)
{
    return ((bucket / ORDER_GROUP) << 24) | (0xffffff - min(b_count, 0xffffff));
}

// Builds one work list.  "a" is the tiled side (queries forward, keys backward),
// "b" the ranged side.
//   FORWARD : b range = keys with pos <= max a pos;  extra = #keys with pos <= min a pos
//   BACKWARD: b range = queries with pos >= min a pos; extra = #queries of the range with pos < max a pos
// STRICT (a key is visible only to later positions, App. B.1's ">" in place of ">="): the
// comparisons with equality swap sides, <= becomes < and >= becomes >.
template <bool FORWARD, bool STRICT>
__device__ void build_list(const int32_t* __restrict__ a_idx, const Searched& b_idx,
                           const int32_t* a_off, const int32_t* b_off, int nb, int tile_a,
                           int tile_b, int n_items_max, int32_t* __restrict__ work_out,
                           long long* counters2, int32_t* s_tile_base, int32_t* s_unit_first, int32_t* s_cost)
{
    // Units (nb <= 256, one thread): a bucket with a tile or more of rows on either side is a
    // unit of its own (its items keep their causal range and mask-free prefix); consecutive buckets
    // that are shorter than a tile on both sides are taken together while their rows on the tiled
    // side fit one tile: only there does one item walk fewer tiles than one item per bucket would.
    // Tiles per unit -> exclusive prefix.
    __shared__ int s_n_units;
    if (threadIdx.x == 0) {
        int acc = 0, u = 0, b = 0;
        while (b < nb) {
            s_unit_first[u] = b;
            s_tile_base[u] = acc;
            int rows = a_off[b + 1] - a_off[b];
            int e = b + 1;
            const bool alone = rows >= tile_a || b_off[b + 1] - b_off[b] >= tile_b;
            while (!alone && e < nb) {
                const int r2 = a_off[e + 1] - a_off[e];
                if (rows + r2 > tile_a || b_off[e + 1] - b_off[e] >= tile_b) break;
                rows += r2;
                ++e;
            }
            acc += (rows + tile_a - 1) / tile_a;
            b = e;
            ++u;
        }
        s_unit_first[u] = nb;
        s_tile_base[u] = acc;
        s_n_units = u;
    }
    __syncthreads();
    const int n_units = s_n_units;
    const int n_items = s_tile_base[n_units];

    auto make_item = [&](int w) -> Item {
        // unit of item w: last u with tile_base[u] <= w
        int lo = 0, hi = n_units - 1;
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (s_tile_base[mid] <= w) lo = mid; else hi = mid - 1;
        }
        const int b = s_unit_first[lo];
        const int b_last = s_unit_first[lo + 1] - 1;
        Item it;
        it.bucket = b;
        it.n_buckets = b_last - b + 1;
        if (b_last > b) {   // several small buckets: all their rows on both sides, every tile tested
            it.a_begin = a_off[b];
            it.a_count = a_off[b_last + 1] - a_off[b];
            it.b_begin = b_off[b];
            it.b_count = b_off[b_last + 1] - b_off[b];
            it.b_extra = FORWARD ? 0 : it.b_count;
            return it;
        }
        it.a_begin = a_off[b] + (w - s_tile_base[lo]) * tile_a;
        it.a_count = min(tile_a, a_off[b + 1] - it.a_begin);
        const int pos_min = a_idx[it.a_begin];
        const int pos_max = a_idx[it.a_begin + it.a_count - 1];
        const int bb = b_off[b], bn = b_off[b + 1] - b_off[b];
        if (FORWARD) {
            it.b_begin = bb;
            it.b_count = count_in<!STRICT>(b_idx, bb, bn, pos_max);
            it.b_extra = count_in<!STRICT>(b_idx, bb, bn, pos_min);
        } else {
            const int first = count_in<STRICT>(b_idx, bb, bn, pos_min);
            it.b_begin = bb + first;
            it.b_count = bn - first;
            it.b_extra = count_in<STRICT>(b_idx, bb, bn, pos_max) - first;
            if (it.b_extra < 0) it.b_extra = 0;
        }
        return it;
    };

    // the first KEEP items of a thread stay in registers between the two passes (their range
    // ends cost dependent memory reads); beyond that they are computed again
    constexpr int KEEP = 4;
    Item kept[KEEP];
    for (int w = threadIdx.x, j = 0; w < n_items; w += RANGES_THREADS, ++j) {
        const Item it = make_item(w);
        s_cost[w] = order_key(it.bucket, it.b_count);
#pragma unroll
        for (int u = 0; u < KEEP; ++u) if (j == u) kept[u] = it;   // register selects, no indexing
    }
    __syncthreads();

    long long tiles = 0, rect = 0;
    for (int w = threadIdx.x, j = 0; w < n_items_max; w += RANGES_THREADS, ++j) {
        if (w < n_items) {
            Item it;
            if (j < KEEP) {
                it = kept[0];
#pragma unroll
                for (int u = 1; u < KEEP; ++u) if (j == u) it = kept[u];
            } else {
                it = make_item(w);
            }
            const int c = order_key(it.bucket, it.b_count);
            // items are generated in bucket order, so those of one bucket pair are a run [lo, hi) of w
            // (binary searches on the pair field); only they have to be compared
            const int pair = c >> 24;
            int lo = 0, hi = w;                      // first item of the pair: in [0, w]
            while (lo < hi) {
                const int m = (lo + hi) >> 1;
                if ((s_cost[m] >> 24) < pair) lo = m + 1; else hi = m;
            }
            int e0 = w + 1, e1 = n_items;            // first item after the pair: in [w + 1, n_items]
            while (e0 < e1) {
                const int m = (e0 + e1) >> 1;
                if ((s_cost[m] >> 24) > pair) e1 = m; else e0 = m + 1;
            }
            hi = e0;
            int rank = lo;
            for (int u = lo; u < hi; ++u) {
                const int cu = s_cost[u];
                rank += (cu < c) || (cu == c && u < w);
            }
            int32_t* o = work_out + (size_t)rank * WORK_STRIDE;
            o[0] = it.a_begin; o[1] = it.a_count; o[2] = it.b_begin; o[3] = it.b_count;
            o[4] = it.b_extra; o[5] = it.bucket; o[6] = it.n_buckets; o[7] = 0;
            tiles += (it.b_count + tile_b - 1) / tile_b;
            rect += (long long)it.a_count * it.b_count;
        } else {
            int32_t* o = work_out + (size_t)w * WORK_STRIDE;
#pragma unroll
            for (int i = 0; i < WORK_STRIDE; ++i) o[i] = 0;
        }
    }
    // block reduction of the two counters
    __shared__ long long s_red[2][RANGES_THREADS / 64];
    for (int off = 32; off > 0; off >>= 1) {
        tiles += __shfl_down(tiles, off);
        rect += __shfl_down(rect, off);
    }
    if ((threadIdx.x & 63) == 0) { s_red[0][threadIdx.x >> 6] = tiles; s_red[1][threadIdx.x >> 6] = rect; }
    __syncthreads();
    if (threadIdx.x == 0 && counters2) {
        long long t = 0, r = 0;
        for (int i = 0; i < RANGES_THREADS / 64; ++i) { t += s_red[0][i]; r += s_red[1][i]; }
        counters2[0] = t; counters2[1] = r;
    }
    __syncthreads();
}

__global__ __launch_bounds__(RANGES_THREADS) void block_ranges_kernel(
    int variant, const int32_t* __restrict__ q_idx, const int32_t* __restrict__ k_idx,
    const int32_t* __restrict__ q_off_g, const int32_t* __restrict__ k_off_g, int T, int nb,
    int fwd_m, int fwd_n, int bwd_n, int bwd_m, int n_fwd, int n_bwd, int stage_shift, int strict,
    int32_t* __restrict__ fwd_work, int32_t* __restrict__ bwd_work, long long* __restrict__ counters)
{
    extern __shared__ int32_t smem[];
    int32_t* s_qoff = smem;                   // [nb+1]
    int32_t* s_koff = s_qoff + nb + 1;        // [nb+1]
    int32_t* s_tile_base = s_koff + nb + 1;   // [nb+1]
    int32_t* s_unit_first = s_tile_base + nb + 1;   // [nb+1]
    const int n_max_items = n_fwd > n_bwd ? n_fwd : n_bwd;
    int32_t* s_cost = s_unit_first + nb + 1;  // [max(n_fwd, n_bwd)]
    int32_t* s_idx = smem + ((4 * (nb + 1) + n_max_items + 3) & ~3);   // [T] when staged, 16-byte aligned
    const int s = blockIdx.x;
    const bool backward = blockIdx.y == 1;
    if (variant == SCFA_QKDROP) {
        if (threadIdx.x == 0) {
            s_qoff[0] = 0; s_qoff[1] = min(max(q_off_g[s], 0), T);
            s_koff[0] = 0; s_koff[1] = min(max(k_off_g[s], 0), T);
        }
    } else {
        for (int b = threadIdx.x; b <= nb; b += RANGES_THREADS) {
            s_qoff[b] = q_off_g[(size_t)s * (nb + 1) + b];
            s_koff[b] = k_off_g[(size_t)s * (nb + 1) + b];
        }
    }
    const int32_t* qi = q_idx + (size_t)s * T;
    const int32_t* ki = k_idx + (size_t)s * T;
    const int32_t* searched_g = backward ? qi : ki;    // the ranged side
    if (stage_shift == 0) {   // 16-byte loads, eight in flight per thread (the segment base is 16-byte aligned when T % 4 == 0)
        if ((T & 3) == 0) {
            const int4* src4 = reinterpret_cast<const int4*>(searched_g);
            int4* dst4 = reinterpret_cast<int4*>(s_idx);
            const int n4 = T >> 2;
            for (int t0 = 0; t0 < n4; t0 += RANGES_THREADS * 8) {
                int4 v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int t = t0 + u * RANGES_THREADS + threadIdx.x;
                    v[u] = t < n4 ? src4[t] : make_int4(0, 0, 0, 0);
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int t = t0 + u * RANGES_THREADS + threadIdx.x;
                    if (t < n4) dst4[t] = v[u];
                }
            }
        } else {
            for (int t = threadIdx.x; t < T; t += RANGES_THREADS) s_idx[t] = searched_g[t];
        }
    } else {                  // every 2^shift-th entry
        const int n_s = ((T - 1) >> stage_shift) + 1;
        for (int i0 = 0; i0 < n_s; i0 += RANGES_THREADS * 8) {   // eight loads in flight per thread
            int32_t v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = i0 + u * RANGES_THREADS + threadIdx.x;
                v[u] = i < n_s ? searched_g[(size_t)i << stage_shift] : 0;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = i0 + u * RANGES_THREADS + threadIdx.x;
                if (i < n_s) s_idx[i] = v[u];
            }
        }
    }
    const Searched searched{searched_g, s_idx, stage_shift};
    __syncthreads();
    long long* cnt = counters ? counters + (size_t)s * 4 : nullptr;
    int32_t* fw = fwd_work + (size_t)s * n_fwd * WORK_STRIDE;
    int32_t* bw = bwd_work ? bwd_work + (size_t)s * n_bwd * WORK_STRIDE : nullptr;
    if (!backward) {
        if (strict) build_list<true, true>(qi, searched, s_qoff, s_koff, nb, fwd_m, fwd_n, n_fwd, fw, cnt, s_tile_base, s_unit_first, s_cost);
        else build_list<true, false>(qi, searched, s_qoff, s_koff, nb, fwd_m, fwd_n, n_fwd, fw, cnt, s_tile_base, s_unit_first, s_cost);
        if (!bwd_work && cnt && threadIdx.x == 0) { cnt[2] = 0; cnt[3] = 0; }
    } else {
        long long* c2 = cnt ? cnt + 2 : nullptr;
        if (strict) build_list<false, true>(ki, searched, s_koff, s_qoff, nb, bwd_n, bwd_m, n_bwd, bw, c2, s_tile_base, s_unit_first, s_cost);
        else build_list<false, false>(ki, searched, s_koff, s_qoff, nb, bwd_n, bwd_m, n_bwd, bw, c2, s_tile_base, s_unit_first, s_cost);
    }
}

int launch_block_ranges(int variant, const int32_t* q_idx, const int32_t* k_idx,
                        const int32_t* q_off, const int32_t* k_off, int S, int T, int nb,
                        int fwd_m, int fwd_n, int bwd_n, int bwd_m, int n_fwd, int n_bwd, int strict,
                        int32_t* fwd_work, int32_t* bwd_work, int64_t* counters, hipStream_t st)
{
    const int n_max = n_fwd > n_bwd ? n_fwd : n_bwd;
    const size_t small = sizeof(int32_t) * ((4 * (size_t)(nb + 1) + (size_t)n_max + 3) & ~(size_t)3);
    int shift = 0;            // the searched vector is staged in LDS whole, or every 2^shift-th entry of it
    while (small + sizeof(int32_t) * ((((size_t)T - 1) >> shift) + 1) > 144 * 1024) ++shift;
    const size_t smem = small + sizeof(int32_t) * ((((size_t)T - 1) >> shift) + 1);
    static std::atomic<unsigned long long> lds_allowed{0};
    { const int rc_ = allow_dynamic_lds(reinterpret_cast<const void*>(&block_ranges_kernel), 144 * 1024, lds_allowed); if (rc_ != SCFA_OK) return rc_; }
    ProfScope prof(SCFA_K_RANGES, st);
    hipLaunchKernelGGL(block_ranges_kernel, dim3(S, bwd_work ? 2 : 1), dim3(RANGES_THREADS), smem, st, variant, q_idx,
                       k_idx, q_off, k_off, T, nb, fwd_m, fwd_n, bwd_n, bwd_m, n_fwd, n_bwd, shift, strict, fwd_work,
                       bwd_work, (long long*)counters);
    SCFA_HIP_TRY(hipGetLastError());
    return SCFA_OK;
}

}  // namespace scfa
