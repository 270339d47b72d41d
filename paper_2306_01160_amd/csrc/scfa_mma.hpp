// Matrix-core and LDS helpers shared by the fp16-compute attention kernels (gfx950).
//
// Compute format.  The permuted Q, K, V (and dO) the kernels consume are fp16: the
// conversion from bf16 is exact for magnitudes in [2^-17, 65504], so scores are the
// same products a bf16 contraction would form, while P and dS -- which must be rounded
// to 16 bits for the second contraction -- keep 11 significant bits instead of 8.
//
// v_mfma_f32_32x32x16_f16 (64 lanes):
//   A (32 x 16): lane l holds row l%32, contraction slots 8*(l/32) .. +7
//   B (16 x 32): lane l holds column l%32, contraction slots 8*(l/32) .. +7
//   C/D (32 x 32): lane l holds column l%32; register i holds row 8*(i/4) + 4*(l/32) + i%4
// Any assignment of contraction indices to slots is valid as long as A and B agree.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace scfa {

using f16x8 = _Float16 __attribute__((ext_vector_type(8)));
using f16x2 = _Float16 __attribute__((ext_vector_type(2)));
using f32x16 = float __attribute__((ext_vector_type(16)));
using i16x4 = short __attribute__((ext_vector_type(4)));

constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

__device__ __forceinline__ f16x8 as_f16x8(uint4 v) { return __builtin_bit_cast(f16x8, v); }

__device__ __forceinline__ f32x16 mfma16(f16x8 a, f16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}

// The same instruction with the accumulator held in the accumulation registers (AccVGPRs), for
// accumulators that live across a whole work item and are only read at its end: they then take no
// architectural VGPRs.  Issued from inline assembly (the compiler would keep a VGPR form); a dependent
// accumulate into the same registers needs no wait, and whoever reads the accumulator afterwards must
// let the last instruction retire (acc_mfma_drain) -- the compiler does not know this statement is a
// matrix instruction.  Not volatile: a pure function of its operands, so LDS reads may be scheduled
// across it.
__device__ __forceinline__ void acc_mfma16(f32x16& acc, f16x8 a, f16x8 b)
{
    asm("s_nop 1\n\tv_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}
// The wait takes the accumulators as operands: every later read of them then depends on it.  (Without them the
// compiler is free to read an accumulator that this statement does not mention before the wait.)
__device__ __forceinline__ void acc_mfma_drain(f32x16& a0, f32x16& a1, f32x16& a2, f32x16& a3, f32x16& a4, f32x16& a5, f32x16& a6,
                                               f32x16& a7)
{
    asm volatile("s_nop 15\n\ts_nop 15" : "+a"(a0), "+a"(a1), "+a"(a2), "+a"(a3), "+a"(a4), "+a"(a5), "+a"(a6), "+a"(a7)::"memory");
}

__device__ __forceinline__ f32x16 zero16()
{
    f32x16 z;
#pragma unroll
    for (int i = 0; i < 16; ++i) z[i] = 0.f;
    return z;
}

// two floats -> packed fp16 pair, round toward zero (finite inputs never become inf)
__device__ __forceinline__ uint32_t pack_f16(float lo, float hi)
{
    return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(lo, hi));
}

// every element of a fragment times c, in fp32, rounded to fp16 (nearest even)
__device__ __forceinline__ f16x8 scale_f16x8(f16x8 v, float c)
{
    f16x8 r;
#pragma unroll
    for (int e = 0; e < 8; ++e) r[e] = (_Float16)((float)v[e] * c);
    return r;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Added to the exponent of every probability that is then truncated to
// fp16: truncation loses half an ulp on average, a relative 2^-11 * E[1/mantissa] = 3.5e-4 for
// log-uniform mantissas; scaling by 1 + 3.5e-4 first (log2 = 5.08e-4) centres the error on zero.
constexpr float RTZ_BIAS_LOG2 = 5.08e-4f;

// makes the compiler treat v as consumed here (pending loads into it are waited for)
template <typename V>
__device__ __forceinline__ void touch(V& v) { asm volatile("" : "+v"(v)); }

// fp32 sum of the two fp16 halves of w, added to acc
__device__ __forceinline__ float add_pair(uint32_t w, float acc)
{
    const f16x2 ones = {(_Float16)1.0f, (_Float16)1.0f};
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, w), ones, acc, false);
}

// exchange between the two lane halves: returns op(x in lanes 0-31, x in lanes 32-63) in all lanes
__device__ __forceinline__ float half_max(float x)
{
    const uint32_t u = __float_as_uint(x);
    auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_sum(float x)
{
    const uint32_t u = __float_as_uint(x);
    auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// registers 8*cc .. 8*cc+7 of an accumulator block as an fp16 B-operand chunk; the
// contraction slots of lane half h are rows { 16*cc + 4h + 0..3, 16*cc + 8 + 4h + 0..3 }
__device__ __forceinline__ f16x8 pack_chunk(const f32x16& p, int cc)
{
    return as_f16x8(make_uint4(pack_f16(p[8 * cc + 0], p[8 * cc + 1]), pack_f16(p[8 * cc + 2], p[8 * cc + 3]),
                               pack_f16(p[8 * cc + 4], p[8 * cc + 5]), pack_f16(p[8 * cc + 6], p[8 * cc + 7])));
}

// ---------------------------------------------------------------------------
// Row-major fp16 tiles in LDS.
//   "rows" operand : contraction along the row (head dimension), one 16-byte read
//   "trans" operand: contraction along the tile's rows; two transposing 8-byte reads
//                    (ds_read_b64_tr_b16) give 4 + 4 consecutive tile rows per lane
// ---------------------------------------------------------------------------
// ds_read_b64_tr_b16 within a block of 16 lanes: lane i receives element i%4 of the four
// 4-element rows addressed by lanes i/4, i/4+4, i/4+8, i/4+12 of its block.
__device__ __forceinline__ uint2 lds_tr_read(const uint16_t* p)
{
    using lds_ptr = i16x4 __attribute__((address_space(3)))*;
    const i16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
    return __builtin_bit_cast(uint2, r);
}

using u32x4 = unsigned int __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------
// Swizzled tiles: row stride D (no padding).  LDS has 64 banks of 4 bytes; a 16-byte read
// is served 16 lanes per cycle and a transposing 8-byte read 32 lanes per cycle, so
//   - 16 consecutive rows reading the same 16-byte chunk (row operand reads), and
//   - 4 consecutive rows reading the same 64 bytes (transposing reads)
// must each land on distinct 16-byte slots of the 256-byte bank line.  The chunk c of row
// r is stored at chunk position c ^ swz(r), with swz chosen per row length so that both hold
// (measured: 4.8 and 2.7 cycles per wavefront instruction against 4 and 2 ideal).
template <int D>
__device__ __forceinline__ int swz(int row)
{
    if (D == 64)   // two rows per bank line: 3 swizzle bits, bit 2 follows row bit 1
        return (((row >> 1) & 1) << 2) | ((row >> 2) & 3);
    // D == 128: one row per bank line: 4 swizzle bits, bits 2-3 follow row bits 0-1
    return ((row & 1) << 2) | (((row >> 1) & 1) << 3) | ((row >> 2) & 3);
}

template <int D>
__device__ __forceinline__ int swz_offset(int row, int col)   // element offset of (row, col) in a tile
{
    return row * D + ((((col >> 3) ^ swz<D>(row)) << 3) | (col & 7));
}

template <int D>
__device__ __forceinline__ f16x8 swz_rows(const uint16_t* tile, int row, int col)
{
    return as_f16x8(*reinterpret_cast<const uint4*>(tile + swz_offset<D>(row, col)));
}

// element offsets of the two transposing reads of lane `lane` for the operand
// A = transpose(tile[r0 .. r0+16)[c0 .. c0+32)): lane l gets column c0 + l%32 and tile rows
// { r0 + 4h + 0..3, r0 + 8 + 4h + 0..3 } (h = l/32), the slot order pack_chunk gives the B operand;
// loop-invariant per lane
template <int D>
__device__ __forceinline__ void swz_trans_offsets(int r0, int c0, int lane, int& off_a, int& off_b)
{
    const int r = lane & 15, blk = (lane >> 4) & 1, h = lane >> 5;
    const int row = r0 + 4 * h + (r >> 2), col = c0 + 16 * blk + 4 * (r & 3);
    off_a = swz_offset<D>(row, col);
    off_b = swz_offset<D>(row + 8, col);
}

__device__ __forceinline__ f16x8 swz_trans(const uint16_t* tile, int off_a, int off_b)
{
    const uint2 a = lds_tr_read(tile + off_a);
    const uint2 b = lds_tr_read(tile + off_b);
    return as_f16x8(make_uint4(a.x, a.y, b.x, b.y));
}

// ---------------------------------------------------------------------------
// Asynchronous tile copies: buffer loads that write straight into LDS (no registers, no
// LDS store instruction).  Lane i of a wavefront's load lands at lds_addr + 16 i, so a
// 64-lane instruction fills 1 KiB of contiguous LDS; the swizzled tile layout is obtained by
// choosing WHICH 16-byte chunk of the global tile each lane fetches.  The loads are issued
// from inline assembly: the compiler then neither counts them nor forces them to complete
// before later LDS reads, and the kernels place the s_waitcnt vmcnt(N) themselves (they are
// the only vector-memory loads in flight inside the tile loops).  Rows past the end of the
// descriptor's range land as zeros.
typedef __attribute__((address_space(3))) unsigned char* lds_byte_ptr;

__device__ __forceinline__ uint32_t lds_address(const void* p)   // byte address inside the workgroup's LDS
{
    return (uint32_t)(uintptr_t)(lds_byte_ptr)(const_cast<void*>(p));
}

// raw buffer descriptor (stride 0, range `bytes`) in scalar registers
__device__ __forceinline__ u32x4 make_desc(const void* base, uint32_t bytes)
{
    const uint64_t a = (uint64_t)(uintptr_t)base;
    u32x4 d;
    d[0] = __builtin_amdgcn_readfirstlane((uint32_t)a);
    d[1] = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32) & 0xffffu);
    d[2] = __builtin_amdgcn_readfirstlane(bytes);
    d[3] = 0x00020000u;
    return d;
}

// lds_addr and soffset must be wave-uniform.  M0 carries the LDS address of the load; the
// compiler flags it as a reserved register in the clobber list, which is the intent here.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void async_load16(u32x4 desc, uint32_t lds_addr, int voffset, int soffset)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :: "s"(lds_addr), "v"(voffset), "s"(desc), "s"(soffset) : "memory", "m0");
}
__device__ __forceinline__ void async_load4(u32x4 desc, uint32_t lds_addr, int voffset, int soffset)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, %3 offen lds"
                 :: "s"(lds_addr), "v"(voffset), "s"(desc), "s"(soffset) : "memory", "m0");
}
#pragma clang diagnostic pop
template <int N>
__device__ __forceinline__ void wait_async()   // at most N asynchronous loads of this wavefront still in flight
{
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}
// every LDS operation of this wavefront done, then the workgroup barrier (no memory fence:
// a fence would make the compiler wait for ALL vector-memory traffic)
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
}

// ROWS contiguous rows x D fp16 of global memory -> swizzled LDS tile (row stride D), by a
// workgroup of THREADS lanes: ROUNDS loads per wavefront.
template <int D, int ROWS, int THREADS>
struct AsyncTile {
    static constexpr int CH = D / 8;                      // 16-byte chunks per row
    static constexpr int ROUNDS = ROWS * CH / THREADS;
    static constexpr int TILE_BYTES = ROWS * D * 2;
    static_assert(ROWS * CH % THREADS == 0, "tile must split evenly over the workgroup");
    int voff[ROUNDS];
    uint32_t wave_off;   // where this wavefront's kilobyte of a round starts: kept in a scalar register, so that the LDS address
                         // of a load (M0) is scalar arithmetic and not a vector add read back with v_readfirstlane per load

    __device__ __forceinline__ void init()
    {
        wave_off = __builtin_amdgcn_readfirstlane(((uint32_t)threadIdx.x >> 6) * 1024u);
#pragma unroll
        for (int u = 0; u < ROUNDS; ++u) {
            const int pos = u * THREADS + (int)threadIdx.x;   // LDS chunk position this lane fills
            const int row = pos / CH, slot = pos % CH;
            voff[u] = (row * CH + (slot ^ swz<D>(row))) * 16;  // the chunk that belongs there
        }
    }
    // one of the ROUNDS loads of a tile, for callers that spread a tile's loads over their own work
    __device__ __forceinline__ void load_round(u32x4 desc, int tile_byte_offset, uint32_t tile_lds, int u) const
    {
        async_load16(desc, tile_lds + wave_off + (uint32_t)(u * THREADS * 16), voff[u], tile_byte_offset);
    }
    // tile_lds: LDS byte address of the tile; tile_byte_offset: wave-uniform offset into the buffer
    __device__ __forceinline__ void load(u32x4 desc, int tile_byte_offset, uint32_t tile_lds) const
    {
#pragma unroll
        for (int u = 0; u < ROUNDS; ++u)
            async_load16(desc, tile_lds + wave_off + (uint32_t)(u * THREADS * 16), voff[u], tile_byte_offset);
    }
};

}  // namespace scfa
