// Device-side building blocks shared by the libgka kernels (gfx950 only).
//
// Everything is organised around the 32x32 MFMA accumulator layout. For a wave64 lane
// l = 32*g + n (g in {0,1}, n in 0..31) and accumulator register r in 0..15, a 32x32 output
// tile holds element (row = kidx(r, g), column = n). The kernels keep one token per lane
// column, so a token's feature vector lives in the registers of its two lanes; a tile of
// such accumulators can be fed back as the B operand of the next MFMA without leaving
// registers, provided the A operand enumerates the contraction index in the same kidx order.
// "Fragment order" below is that order: fragment (.., blk, h) lane (n, g) element p holds the
// matrix entry at row n and column 32*blk + kidx(h*VEC + p, g).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "gka_kernels.hpp"

namespace gka {

constexpr float kMinLog2Gate = -144.269504f;   // log2 of the smallest gate, exp(-100)

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint16_t u16x4 __attribute__((ext_vector_type(4)));
typedef uint16_t u16x8 __attribute__((ext_vector_type(8)));

// Row (contraction index within a 32-block) of accumulator register r on lane half g.
__device__ __forceinline__ constexpr int kidx(int r, int g) { return 8 * (r >> 2) + 4 * g + (r & 3); }

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// Round to nearest even, as the hardware conversion does.
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float x)
{
    __bf16 h = (__bf16)x;
    return __builtin_bit_cast(uint16_t, h);
}

// ---- tensor element types of q, k, v, o ---------------------------------------------------
struct IOF32 {
    typedef float type;
    static __device__ __forceinline__ float load(const void *p, int64_t i) { return ((const float *)p)[i]; }
    // four consecutive elements, 16-byte aligned
    static __device__ __forceinline__ f32x4 load4(const void *p, int64_t i) { return *(const f32x4 *)((const float *)p + i); }
    // the same without conversion, so that the load stays asynchronous until its first use
    typedef f32x4 raw4;
    static __device__ __forceinline__ raw4 load_raw4(const void *p, int64_t i) { return load4(p, i); }
    static __device__ __forceinline__ f32x4 cvt4(raw4 r) { return r; }
    static __device__ __forceinline__ void store4(void *p, int64_t i, float a, float b, float c, float d)
    {
        f32x4 v = {a, b, c, d};
        *(f32x4 *)((float *)p + i) = v;
    }
    static __device__ __forceinline__ void store1(void *p, int64_t i, float a) { ((float *)p)[i] = a; }
};
struct IOBF16 {
    typedef uint16_t type;
    static __device__ __forceinline__ float load(const void *p, int64_t i)
    {
        return bf16_bits_to_f32(((const uint16_t *)p)[i]);
    }
    // four consecutive elements, 8-byte aligned
    static __device__ __forceinline__ f32x4 load4(const void *p, int64_t i)
    {
        return cvt4(load_raw4(p, i));
    }
    // the same without conversion, so that the load stays asynchronous until its first use
    typedef u16x4 raw4;
    static __device__ __forceinline__ raw4 load_raw4(const void *p, int64_t i)
    {
        return *(const u16x4 *)((const uint16_t *)p + i);
    }
    static __device__ __forceinline__ f32x4 cvt4(raw4 b)
    {
        f32x4 v = {bf16_bits_to_f32(b[0]), bf16_bits_to_f32(b[1]), bf16_bits_to_f32(b[2]), bf16_bits_to_f32(b[3])};
        return v;
    }
    static __device__ __forceinline__ void store4(void *p, int64_t i, float a, float b, float c, float d)
    {
        u16x4 v = {f32_to_bf16_bits(a), f32_to_bf16_bits(b), f32_to_bf16_bits(c), f32_to_bf16_bits(d)};
        *(u16x4 *)((uint16_t *)p + i) = v;
    }
    static __device__ __forceinline__ void store1(void *p, int64_t i, float a)
    {
        ((uint16_t *)p)[i] = f32_to_bf16_bits(a);
    }
};

// Row-major LDS tiles of k or v rows (features contiguous) come in two layouts, both a functor (row, col) ->
// element offset: rows padded so that consecutive rows start 32 bytes apart modulo 256, or unpadded rows whose
// 32-byte granules are XOR-swizzled with the row number. Either way the four rows addressed by a 16-lane block of
// a transpose read (below) fall into disjoint banks.
struct PaddedRows {
    int rs;                                        // elements per row including the padding
    __device__ __forceinline__ int operator()(int row, int col) const { return row * rs + col; }
};
template <int ROW_BYTES, int ELEM_BYTES>
struct SwizzledRows {
    static constexpr int kGranules = ROW_BYTES / 32;
    static constexpr int kMask = (kGranules < 8 ? kGranules : 8) - 1;
    __device__ __forceinline__ int operator()(int row, int col) const
    {
        const int byte = col * ELEM_BYTES;
        return (row * ROW_BYTES + (byte ^ ((row & kMask) << 5))) / ELEM_BYTES;
    }
};

// Transposed operand fragment from a row-major LDS tile: the VEC elements x[tok_of(p)][col] of this lane.
// Generic version: one LDS read per element.
template <class MMA, class Layout, class TokOf>
__device__ __forceinline__ typename MMA::frag gather_transposed(const typename MMA::elem_t *tile, Layout at, int col,
                                                                TokOf tok_of)
{
    typename MMA::elem_t e[MMA::VEC];
#pragma unroll
    for (int p = 0; p < MMA::VEC; ++p) e[p] = tile[at(tok_of(p), col)];
    return MMA::pack_elems(e);
}

// bf16 fast path for fragments whose 8 tokens are two runs of 4 consecutive tokens (t0 .. t0+3, t1 .. t1+3):
// two ds_read_b64_tr_b16 transpose reads. Within each block of 16 lanes the instruction hands lane i the four
// 16-bit values found at element (i % 4) of the addresses supplied by lanes (i / 4), (i / 4) + 4, + 8, + 12 of
// the block. So lane i supplies the address of token run[i / 4] at the 4-column group (i % 4) of its block's 16
// columns, and receives tokens run[0..3] at its own column. `col16` is the first of the block's 16 columns.
template <class Layout>
__device__ __forceinline__ bf16x8 gather_transposed_bf16(const uint16_t *tile, Layout at, int col16, int lane, int t0,
                                                         int t1)
{
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    const int i = lane & 15;
    const uint16_t *p0 = tile + at(t0 + (i >> 2), col16 + 4 * (i & 3));
    const uint16_t *p1 = tile + at(t1 + (i >> 2), col16 + 4 * (i & 3));
    s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)p0);
    s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)p1);
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    s16x8 r = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
    return __builtin_bit_cast(bf16x8, r);
}

// The same two transpose reads written as assembly, including the wait for their data. The compiler orders every
// LDS read it knows of behind all copies into LDS (below) that are in flight, whichever part of LDS they fill; a
// read it does not see is not held back. For tiles that no copy in flight writes to.
template <class Layout>
__device__ __forceinline__ bf16x8 gather_transposed_bf16_untracked(const uint16_t *tile, Layout at, int col16, int lane,
                                                                   int t0, int t1)
{
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) const uint16_t lds_u16;
    const int i = lane & 15;
    const uint32_t p0 = (uint32_t)(uintptr_t)(lds_u16 *)(tile + at(t0 + (i >> 2), col16 + 4 * (i & 3)));
    const uint32_t p1 = (uint32_t)(uintptr_t)(lds_u16 *)(tile + at(t1 + (i >> 2), col16 + 4 * (i & 3)));
    u32x2 a, b;
    asm volatile("ds_read_b64_tr_b16 %0, %2\n\tds_read_b64_tr_b16 %1, %3\n\ts_waitcnt lgkmcnt(0)"
                 : "=&v"(a), "=&v"(b)
                 : "v"(p0), "v"(p1)
                 : "memory");
    const u32x4 r = {a[0], a[1], b[0], b[1]};
    return __builtin_bit_cast(bf16x8, r);
}

// Asynchronous copy global -> LDS without staging registers: every lane moves 16 bytes, a wave's 64 pieces land
// contiguously at the (wave-uniform) destination. Completion is tracked by the vector-memory counter: wait for it
// (s_waitcnt vmcnt) and pass a barrier before other waves read the data. The copies are buffer loads: a
// descriptor over the source (wave-uniform base) and a 32-bit byte offset per lane. (The flat form of the same
// copy makes the compiler turn every later vector-memory wait of the wave into a full drain.)
typedef __amdgpu_buffer_rsrc_t buffer_rsrc;
__device__ __forceinline__ buffer_rsrc make_raw_buffer(const void *base)
{
    return __builtin_amdgcn_make_buffer_rsrc((void *)base, 0, 0x7fffffff, 0x00020000);
}
__device__ __forceinline__ void async_copy16_to_lds(void *lds_wave_base, buffer_rsrc src, int lane_byte_offset,
                                                    int wave_byte_offset)
{
    __builtin_amdgcn_raw_ptr_buffer_load_lds(src, (__attribute__((address_space(3))) void *)lds_wave_base, 16,
                                             lane_byte_offset, wave_byte_offset, 0, 0);
}
__device__ __forceinline__ void wait_all_memory() { __builtin_amdgcn_s_waitcnt(0); }

// The same copy as an assembly statement, which the compiler does not track: it neither orders later LDS accesses
// of the wave behind it (for a copy it knows of it does, whichever part of LDS they touch) nor counts it in the
// vector-memory waits it inserts (those then wait for more than they need, never for less: the counter retires in
// issue order). The caller waits for the copy itself, with wait_vector_memory_but<N> where at least N vector-memory
// instructions of the wave are certain to follow it, and passes a barrier before other waves read the data.
// `rsrc`: the four words of a raw buffer descriptor over the source (wave-uniform); `lds_wave_addr`: LDS byte
// address of the wave's 1 KiB destination (wave-uniform; it travels through M0).
typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ i32x4 raw_buffer_words(const void *base)
{
    const uint64_t b = (uint64_t)(uintptr_t)base;
    return i32x4{(int32_t)(uint32_t)b, (int32_t)((uint32_t)(b >> 32) & 0xffffu), 0x7fffffff, 0x00020000};
}
__device__ __forceinline__ void async_copy16_to_lds_untracked(uint32_t lds_wave_addr, i32x4 rsrc, int lane_byte_offset)
{
    // (M0 is put back: the compiler does not take a clobber of it into account)
    uint32_t saved_m0;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\t"
                 "buffer_load_dwordx4 %2, %3, 0 offen lds\n\ts_mov_b32 m0, %0"
                 : "=&s"(saved_m0)
                 : "s"(lds_wave_addr), "v"(lane_byte_offset), "s"(rsrc)
                 : "memory");
}
// At most N vector-memory instructions of this wave are still outstanding: everything issued before the last N has
// completed.
template <int N>
__device__ __forceinline__ void wait_vector_memory_but()
{
    static_assert(N >= 0 && N < 64, "the counter holds 6 bits");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Workgroup barrier that orders LDS traffic only: this wave's LDS operations have completed (lgkmcnt(0)), then
// s_barrier. Unlike __syncthreads() it carries no global-memory fence, so vector-memory loads that are still in
// flight (prefetches for later steps) are not waited for.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// ---- arithmetic of the matrix products ------------------------------------------------------
// VEC = operand elements per lane per MFMA; HS = MFMA steps per 32-block of the contraction.
struct MmaBF16 {
    static constexpr int VEC = 8;
    static constexpr int HS = 2;
    static constexpr bool kSplitReadout = true;   // readout uses hi+lo operands
    // P and the state product of a pass share one sweep over delta, and part of the update is pinned between the
    // MFMAs of the intra-chunk product
    static constexpr bool kFusedPassSweep = true;
    typedef bf16x8 frag;
    typedef uint16_t elem_t;                      // operand element as stored in LDS rows
    // Padding of a row-major LDS tile (elements): rows 32 bytes apart modulo 256, so that the four rows
    // addressed by a 16-lane block of a transpose read fall into disjoint banks.
    static constexpr int kRowPad = 16;
    static __device__ __forceinline__ elem_t to_elem(float x) { return f32_to_bf16_bits(x); }
    static __device__ __forceinline__ float from_elem(elem_t e) { return bf16_bits_to_f32(e); }
    // fragment from VEC stored elements
    static __device__ __forceinline__ frag pack_elems(const elem_t *e)
    {
        u16x8 u = {e[0], e[1], e[2], e[3], e[4], e[5], e[6], e[7]};
        return __builtin_bit_cast(frag, u);
    }
    static __device__ __forceinline__ void store4(elem_t *dst, f32x4 v)
    {
        u16x4 u = {f32_to_bf16_bits(v[0]), f32_to_bf16_bits(v[1]), f32_to_bf16_bits(v[2]), f32_to_bf16_bits(v[3])};
        *(u16x4 *)dst = u;
    }
    static __device__ __forceinline__ f32x16 mma(frag a, frag b, f32x16 c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
    // operand fragment from VEC consecutive float values
    static __device__ __forceinline__ frag pack(const float *x)
    {
        frag f;
#pragma unroll
        for (int p = 0; p < VEC; ++p) f[p] = (__bf16)x[p];
        return f;
    }
    static __device__ __forceinline__ float elem(frag f, int p) { return (float)f[p]; }
    // all VEC elements as floats: one shift or mask per element of the packed words
    static __device__ __forceinline__ void unpack(frag f, float *x)
    {
        typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
        const u32x4 wds = __builtin_bit_cast(u32x4, f);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[2 * i] = __uint_as_float(wds[i] << 16);
            x[2 * i + 1] = __uint_as_float(wds[i] & 0xffff0000u);
        }
    }
    static __device__ __forceinline__ frag zero()
    {
        frag f;
#pragma unroll
        for (int p = 0; p < VEC; ++p) f[p] = (__bf16)0.0f;
        return f;
    }
};
struct MmaF32 {
    static constexpr int VEC = 1;
    static constexpr int HS = 16;
    static constexpr bool kSplitReadout = false;
    // 64 contraction steps per sweep and 64 MFMAs per intra-chunk product: the fused sweep's staggered reads and a
    // pinned interleaving cost more than they save
    static constexpr bool kFusedPassSweep = false;
    typedef float frag;
    typedef float elem_t;
    static constexpr int kRowPad = 4;
    static __device__ __forceinline__ elem_t to_elem(float x) { return x; }
    static __device__ __forceinline__ float from_elem(elem_t e) { return e; }
    static __device__ __forceinline__ frag pack_elems(const elem_t *e) { return e[0]; }
    static __device__ __forceinline__ void store4(elem_t *dst, f32x4 v) { *(f32x4 *)dst = v; }
    static __device__ __forceinline__ f32x16 mma(frag a, frag b, f32x16 c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ frag pack(const float *x) { return x[0]; }
    static __device__ __forceinline__ float elem(frag f, int) { return f; }
    static __device__ __forceinline__ void unpack(frag f, float *x) { x[0] = f; }
    static __device__ __forceinline__ frag zero() { return 0.0f; }
};

__device__ __forceinline__ f32x16 zero16()
{
    f32x16 z;
#pragma unroll
    for (int i = 0; i < 16; ++i) z[i] = 0.0f;
    return z;
}

// Inclusive prefix sum over the 64 lanes of a wave with DPP moves: shifts by 1, 2, 4, 8 inside each row of 16
// lanes (lanes shifted in from outside the row contribute 0), then the last lane of row 0 / row 2 is broadcast into
// row 1 / row 3, then lane 31 into rows 2 and 3.
__device__ __forceinline__ float wave_inclusive_scan(float x, int /*lane*/)
{
    auto dpp_add = [](float v, auto ctrl, auto row_mask) {
        const int moved = __builtin_amdgcn_update_dpp(0, __float_as_int(v), decltype(ctrl)::value,
                                                      decltype(row_mask)::value, 0xf, false);
        return v + __int_as_float(moved);
    };
    x = dpp_add(x, std::integral_constant<int, 0x111>{}, std::integral_constant<int, 0xf>{});   // row_shr:1
    x = dpp_add(x, std::integral_constant<int, 0x112>{}, std::integral_constant<int, 0xf>{});   // row_shr:2
    x = dpp_add(x, std::integral_constant<int, 0x114>{}, std::integral_constant<int, 0xf>{});   // row_shr:4
    x = dpp_add(x, std::integral_constant<int, 0x118>{}, std::integral_constant<int, 0xf>{});   // row_shr:8
    x = dpp_add(x, std::integral_constant<int, 0x142>{}, std::integral_constant<int, 0xa>{});   // row_bcast:15 -> rows 1, 3
    x = dpp_add(x, std::integral_constant<int, 0x143>{}, std::integral_constant<int, 0xc>{});   // row_bcast:31 -> rows 2, 3
    return x;
}

// Value of x on a lane known at compile time or wave-uniform (no LDS crossbar involved).
__device__ __forceinline__ float lane_value(float x, int src_lane)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), src_lane));
}

__device__ __forceinline__ float wave_sum(float x)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
    return x;
}

// log2(gamma) with the documented floor. Decays are kept in base-2 log space (the hardware's exp and log are
// base 2): cumulative sums of these, and exp2 of their differences.
__device__ __forceinline__ float log2_gate(float gamma) { return fmaxf(log2f(gamma), kMinLog2Gate); }

}  // namespace gka
