// Device code of the 128 x 128 owner-workgroup kernel (templates; instantiated one instance per
// translation unit, see gemm_owner_*.hip) and the helpers it shares with the 256 x 256 kernels.
//
// One workgroup (256 threads = 4 waves as 2 x 2) owns a region of one C tile for the whole
// reduction: it walks the reduction tiles L = 0..KT-1 in ascending order, runs each tile product
// A(I,L)*B(L,J) on the matrix cores at that task's precision q, and writes C once.  Nothing else
// ever touches that region, so there are no atomics and the result is reproducible.  Regions
// are 128 x 128 (gemm_mp_owner_kernel: instances for FP64 and for FP32 C tiles, with and without
// the two options described below), or
// 256 x 256 for FP32 C tiles whose products are all FP8 x FP8, all MXFP8 x MXFP8 or all
// MXFP4 x MXFP4 (gemm_mp_fp8_region_kernel, at the end of this file).
//
// Data path of one reduction chunk (128 bytes of converted reduction index per row, i.e.
// 16 FP64 / 32 FP32 / 64 FP16 / 128 FP8 values) in the 128 x 128 kernels:
//   FP64 / FP32 products: global (stored precision) -> registers -> convert to q ("receiver-side
//   conversion": exact up-casts with the tile's 2^e applied, or the one down-cast FP64 -> FP32)
//   -> LDS (unpadded rows, 16-byte segments swizzled) -> 16x16 MFMA fragments.  The loads of
//   the next chunk are issued under the MFMAs of the current one and land in the other LDS
//   stage; the stream runs across tile-product boundaries so the pipeline never drains inside
//   a C region.
//   FP16 / FP8 products whose operands need no conversion skip the registers:
//   global -> LDS by buffer-load-to-LDS into a ring of five unpadded, swizzled stages.
//   FP16 products with an operand stored in FP8: in the MIXED instances (launched when such
//   products exist) the FP8 operand takes the ring as it is and is converted between the
//   fragment read and the MFMA; in the others a two-stage loop with conversion in registers on
//   the way to LDS, rows padded by 8 B.
//   BF16 products (BF instances, launched when A or B has BF16 tiles): the FP16 ring with the
//   BF16 matrix instruction and, for an FP8 operand, the BF16 form of the conversion; marked by
//   a flag in the product's table record.
//
// Fragment convention.  Packed A tiles are row-major and packed B tiles are stored transposed,
// so both operands have the reduction index contiguous.  Which reduction index a lane's bytes
// are does not matter as long as A and B agree, and they do by construction.  The accumulator
// of a 16x16 FP32-result MFMA holds C[4g+v][i] in register v (i = lane%16, g = lane/16); the
// FP64 MFMA holds C[4v+g][i], so on the FP64 path lane i reads A row 4*(i%4) + i/4 instead of
// row i, which makes both accumulator kinds address the same C element in the same lane and
// register.
#pragma once
#include <type_traits>
#include <utility>

#include "gemm_mp_internal.h"

namespace gmp {


typedef double d4 __attribute__((ext_vector_type(4)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h2v __attribute__((ext_vector_type(2)));
typedef __bf16 bf2v __attribute__((ext_vector_type(2)));
typedef int i8v __attribute__((ext_vector_type(8)));
typedef float f2v __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // native vectors: these stay in registers
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kRowBytes = 128;                       // converted bytes per row and chunk
constexpr int kRowStride = 136;                      // padded stages (two-stage FP16 / FP8 loop): + 8 B,
                                                     // 17 eight-byte words per row, so the 16 rows x 4
                                                     // k-groups of a fragment read and the 8 rows x 8
                                                     // parts of a staging write spread over the banks
constexpr int kOperandStage = kMacro * kRowStride;   // 17408 B: operand pitch of padded and of swizzled stages
constexpr int kStage = 2 * kOperandStage;            // A then B
constexpr int kHiLdsBytes = 2 * kStage;              // two stages, 69632 B

// FP16 / FP8 products use a ring of five stages of unpadded 128-byte rows whose 16-byte slots
// are XOR-swizzled with (row & 7): slot = segment ^ (row & 7).
constexpr int kLoOperand = kMacro * kRowBytes;       // 16384 B
constexpr int kLoStage = 2 * kLoOperand;             // A then B: 32768 B
constexpr int kLoStages = 5;                         // chunk i lives in stage i % 5, requested 4 chunks ahead
constexpr int kLoLdsBytes = kLoStages * kLoStage;    // 163840 B: all of the LDS of a CU
constexpr int kLdsBytes = kLoLdsBytes > kHiLdsBytes ? kLoLdsBytes : kHiLdsBytes;
constexpr int kThreads = 256;

enum { Q64 = GEMM_MP_FP64, Q32 = GEMM_MP_FP32, Q16 = GEMM_MP_FP16, Q8 = GEMM_MP_FP8_E4M3 };

// Raw (still in stored precision) data of one 16-byte converted segment.  Every segment is
// fetched with the same instruction whatever the stored precision: the aligned 16 bytes that
// contain its source (plus the next 16 for the one down-cast, FP64 -> FP32, whose source is
// 32 bytes).  Loads therefore need no control flow and no per-chunk address arithmetic in the
// vector ALU: they are buffer loads whose descriptor is the packed tile, whose vector offset
// is a per-thread constant of the tile product, and whose scalar offset carries the chunk and
// the row block.  When the source is narrower than 16 bytes, neighbouring lanes fetch the same
// 16 bytes and each picks its part at conversion time (`sub` = byte offset of its source
// inside them).  This matters on gfx950: FP64 and FP32 MFMAs do not overlap with other vector
// ALU instructions, so every one of those in the inner loop costs matrix throughput.
struct Raw { u32x4 lo, hi; };

// One operand tile of a tile product.  Everything is wave-uniform except voff and sub.
struct Operand {
    const char *base;              // the packed tile and its size: the buffer descriptor is
    int bytes;                     // formed from them at each load (scalar moves only)
    int p, e;                      // stored precision, scale exponent
    int voff;                      // this thread's first segment in chunk 0, aligned down to 16 B
    int sub;                       // offset of that segment's source inside the 16 loaded bytes; from bit 8 up the
                                   // variant of the format that p does not tell (kept in this per-lane register
                                   // because scalar registers are the scarce ones): 1 = p is Q16 and the tile holds
                                   // BF16 numbers (no scale), 2 / 3 = p is Q8 and the tile is MXFP8 / MXFP4 (one
                                   // scale byte per block of 32 behind the elements).  Only the loop for such
                                   // operands under FP64 / FP32 products (product_loop_widening) ever sees these bits.
};

// One tile product A(I,L)*B(L,J): q is its precision (-1: there is none).
struct Product {
    Operand a, b;
    int q;
};

// soff: byte offset of (chunk, row block) in the tile; down: FP64 tile feeding an FP32 product.
__device__ __forceinline__ void load_seg(Raw &r, const Operand &o, int soff, bool down)
{
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)o.base, 0, o.bytes, 0x00020000);
    r.lo = __builtin_amdgcn_raw_buffer_load_b128(rsrc, o.voff, soff, 0);
    if (down) r.hi = __builtin_amdgcn_raw_buffer_load_b128(rsrc, o.voff + 16, soff, 0);
}

__device__ __forceinline__ float half_lo(uint32_t w) { return (float)__builtin_bit_cast(_Float16, (unsigned short)(w & 0xffffu)); }
__device__ __forceinline__ float half_hi(uint32_t w) { return (float)__builtin_bit_cast(_Float16, (unsigned short)(w >> 16)); }
__device__ __forceinline__ uint32_t pack_half2(float a, float b)
{
    return (uint32_t)__builtin_bit_cast(unsigned short, (_Float16)a) |
           ((uint32_t)__builtin_bit_cast(unsigned short, (_Float16)b) << 16);
}
__device__ __forceinline__ u32x2 dbits(double d) { return __builtin_bit_cast(u32x2, d); }
__device__ __forceinline__ double as_double(uint32_t lo, uint32_t hi) { return __builtin_bit_cast(double, u32x2{lo, hi}); }
__device__ __forceinline__ uint32_t pick_word(const u32x4 v, int w)      // w = 0..3, per lane
{
    const uint32_t a = (w & 1) ? v.y : v.x, b = (w & 1) ? v.w : v.z;
    return (w & 2) ? b : a;
}
__device__ __forceinline__ u32x2 pick_pair(const u32x4 v, int hi)         // low or high 8 bytes
{
    return u32x2{hi ? v.z : v.x, hi ? v.w : v.y};
}

// Receiver-side conversion of one segment to precision Q.  e: the tile's scale exponent;
// sub: byte offset of the segment's source inside the 16 bytes that were loaded.
template <int Q>
__device__ __forceinline__ u32x4 convert(const Raw &r, int p, int e, int sub)
{
    u32x4 o = r.lo;
    if (Q == Q64) {
        if (p == Q64) return o;
        double a, b;
        if (p == Q32) {
            const u32x2 w = pick_pair(r.lo, sub >> 3);
            a = (double)__uint_as_float(w.x); b = (double)__uint_as_float(w.y);
        } else if (p == Q16) {
            const uint32_t w = pick_word(r.lo, sub >> 2);
            a = ldexp((double)half_lo(w), e); b = ldexp((double)half_hi(w), e);
        } else {
            const uint32_t w = pick_word(r.lo, sub >> 2) >> ((sub & 2) * 8);
            a = ldexp((double)__builtin_amdgcn_cvt_f32_fp8((int)w, 0), e);
            b = ldexp((double)__builtin_amdgcn_cvt_f32_fp8((int)w, 1), e);
        }
        const u32x2 ab = dbits(a), bb = dbits(b);
        o.x = ab.x; o.y = ab.y; o.z = bb.x; o.w = bb.y;
    } else if (Q == Q32) {
        if (p == Q32) return o;
        float f0, f1, f2, f3;
        if (p == Q64) {        // the only down-cast: round to nearest even
            f0 = (float)as_double(r.lo.x, r.lo.y);
            f1 = (float)as_double(r.lo.z, r.lo.w);
            f2 = (float)as_double(r.hi.x, r.hi.y);
            f3 = (float)as_double(r.hi.z, r.hi.w);
        } else if (p == Q16) {
            const u32x2 w = pick_pair(r.lo, sub >> 3);
            f0 = ldexpf(half_lo(w.x), e); f1 = ldexpf(half_hi(w.x), e);
            f2 = ldexpf(half_lo(w.y), e); f3 = ldexpf(half_hi(w.y), e);
        } else {
            const int w = (int)pick_word(r.lo, sub >> 2);
            f0 = ldexpf(__builtin_amdgcn_cvt_f32_fp8(w, 0), e);
            f1 = ldexpf(__builtin_amdgcn_cvt_f32_fp8(w, 1), e);
            f2 = ldexpf(__builtin_amdgcn_cvt_f32_fp8(w, 2), e);
            f3 = ldexpf(__builtin_amdgcn_cvt_f32_fp8(w, 3), e);
        }
        o.x = __float_as_uint(f0); o.y = __float_as_uint(f1); o.z = __float_as_uint(f2); o.w = __float_as_uint(f3);
    } else if (Q == Q16) {
        if (p == Q16) return o;
        // FP8 -> FP16 is exact (every e4m3 number is a binary16 number); operands stay scaled
        const u32x2 w = pick_pair(r.lo, sub >> 3);
        const int w0 = (int)w.x, w1 = (int)w.y;
        o.x = pack_half2(__builtin_amdgcn_cvt_f32_fp8(w0, 0), __builtin_amdgcn_cvt_f32_fp8(w0, 1));
        o.y = pack_half2(__builtin_amdgcn_cvt_f32_fp8(w0, 2), __builtin_amdgcn_cvt_f32_fp8(w0, 3));
        o.z = pack_half2(__builtin_amdgcn_cvt_f32_fp8(w1, 0), __builtin_amdgcn_cvt_f32_fp8(w1, 1));
        o.w = pack_half2(__builtin_amdgcn_cvt_f32_fp8(w1, 2), __builtin_amdgcn_cvt_f32_fp8(w1, 3));
    }
    return o;
}

struct Geometry {
    bool ring;                      // pure FP16 / FP8 products go through the DMA ring (set in every kernel instance)
    int tid, lane, li, g, wm, wn;
    int seg_row, seg_part;          // staging: this thread's first row and its 16-byte part
    int wbase;                      // byte offset of that segment in a padded LDS operand stage
    int wsw;                        // the same in a swizzled stage (FP64 / FP32 products)
};

struct Region {
    int nb, arow0, brow0;
    int kt_eff;                     // number of reduction tiles to process (0 when alpha == 0)
    const ProductDesc *prod;        // this C tile's row of the product table: entry L
};

// FP16 / FP8 products whose operands are both stored in the product's precision run through the
// DMA ring (lo_run); in the kernel instance built with MIXED so do FP16 products one of whose
// operands is stored in FP8; every other product expects its first chunk staged by its
// predecessor.  ring_mix: which operand of an FP16 product is stored in FP8 (0 none, 1 A, 2 B).
__device__ __forceinline__ int ring_mix(int q, int pa, int pb) { return q != Q16 ? 0 : pa == Q8 ? 1 : pb == Q8 ? 2 : 0; }
template <bool MIXED>
__device__ __forceinline__ bool is_ring(const Product &pr, const Geometry &G)
{
    if constexpr (MIXED) {
        if (pr.q == Q8) return pr.a.p == Q8 && pr.b.p == Q8;
        return pr.q == Q16 && (pr.a.p == Q16 || pr.b.p == Q16);
    } else {
        return G.ring && (pr.q == Q16 || pr.q == Q8) && pr.a.p == pr.q && pr.b.p == pr.q;
    }
}
// An FP64 / FP32 product one of whose operands is a BF16, MXFP8 or MXFP4 tile: such tiles are
// widened on the receiving side by a loop of their own (product_loop_widening), which also stages
// its own first chunk, so that the staging code of every other product stays what it is.
__device__ __forceinline__ bool is_widening(const Product &pr)
{
    return pr.q >= 0 && pr.q <= Q32 && __builtin_amdgcn_readfirstlane((pr.a.sub | pr.b.sub) >> 8) != 0;
}
template <bool MIXED>
__device__ __forceinline__ bool wants_first_chunk(const Product &pr, const Geometry &G)
{
    return pr.q >= 0 && !is_ring<MIXED>(pr, G) && !is_widening(pr);
}


__device__ __forceinline__ int chunk_elems(int q) { return kRowBytes >> (3 - q); }   // 16, 32, 64, 128

// Nothing may be moved across this point by the instruction scheduler.
#define SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

// The per-lane values every loop works with, from the thread index.
__device__ __forceinline__ Geometry make_geometry(int tid, bool ring)
{
    Geometry G;
    G.ring = ring;
    G.tid = tid;
    G.lane = tid & 63;
    G.li = G.lane & 15;
    G.g = G.lane >> 4;
    const int wave = tid >> 6;
    G.wm = wave >> 1;
    G.wn = wave & 1;
    G.seg_row = tid >> 3;
    G.seg_part = tid & 7;
    G.wbase = G.seg_row * kRowStride + G.seg_part * 16;
    G.wsw = G.seg_row * kRowBytes + ((G.seg_part ^ ((G.seg_row >> 1) & 7)) * 16);
    return G;
}

// A copy of the lane geometry whose values the optimiser must treat as new.  Every product
// loop starts from one: otherwise the per-lane addresses of all the specialised loops are
// hoisted to the top of the kernel and held in registers for its whole life, which pushes the
// staging data of the inner loops out of the vector registers.
__device__ __forceinline__ Geometry fresh(const Geometry &G)
{
    Geometry g = G;
    asm volatile("" : "+v"(g.li), "+v"(g.g), "+v"(g.wm), "+v"(g.wn), "+v"(g.wbase), "+v"(g.wsw), "+v"(g.seg_row), "+v"(g.seg_part));
    return g;
}

// Staging of one chunk: each thread owns four 16-byte converted segments per operand
// (rows seg_row + 32 j, bytes [16 part, 16 part + 16) of the row).  c: chunk index in the product.
__device__ __forceinline__ void load_pair(Raw &ra, Raw &rb, const Product &pr, int nb, int c, int j)
{
    // element offset of (chunk c, row block j) in a tile, then bytes in each operand's precision
    const int eoff = c * chunk_elems(pr.q) + j * 32 * nb;
    load_seg(ra, pr.a, eoff << (3 - pr.a.p), pr.q == Q32 && pr.a.p == Q64);
    load_seg(rb, pr.b, eoff << (3 - pr.b.p), pr.q == Q32 && pr.b.p == Q64);
}

__device__ __forceinline__ void lds_store16(char *p, u32x4 v)     // rows are only 8-byte aligned
{
    *(u32x2 *)p = u32x2{v.x, v.y};
    *(u32x2 *)(p + 8) = u32x2{v.z, v.w};
}

// Two LDS layouts of an operand stage (128 rows of 128 converted bytes):
//  - FP16 / FP8 products outside the ring: rows padded to 136 bytes;
//  - FP64 / FP32 products: rows unpadded, the 16-byte segment s of row r stored in slot
//    s ^ ((r >> 1) & 7).  Stores and fragment reads are then whole aligned 16-byte accesses
//    (half as many instructions as with 8-byte ones, and every offset fits the instructions'
//    immediate field: FP64 / FP32 MFMAs do not overlap with the vector ALU, so each address
//    add saved is matrix time won), and both are free of bank conflicts: the sixteen lanes
//    served together read sixteen consecutive rows, whose slots are distinct modulo 256 bytes.
template <int Q>
__device__ __forceinline__ void store_pair(const Raw &ra, const Raw &rb, const Product &pr, const Geometry &G, char *stage, int j)
{
    if constexpr (Q == Q64 || Q == Q32) {
        char *dst = stage + G.wsw + j * (32 * kRowBytes);
        *(u32x4 *)dst = convert<Q>(ra, pr.a.p, pr.a.e, pr.a.sub);
        *(u32x4 *)(dst + kOperandStage) = convert<Q>(rb, pr.b.p, pr.b.e, pr.b.sub);
    } else {
        char *dst = stage + G.wbase + j * (32 * kRowStride);
        lds_store16(dst, convert<Q>(ra, pr.a.p, pr.a.e, pr.a.sub));
        lds_store16(dst + kOperandStage, convert<Q>(rb, pr.b.p, pr.b.e, pr.b.sub));
    }
}

// The same for a product whose precision is only known at run time (the next tile product).
__device__ __forceinline__ void store_pair_any(const Raw &ra, const Raw &rb, const Product &pr, const Geometry &G, char *stage, int j)
{
    switch (pr.q) {
    case Q64: store_pair<Q64>(ra, rb, pr, G, stage, j); break;
    case Q32: store_pair<Q32>(ra, rb, pr, G, stage, j); break;
    case Q16: store_pair<Q16>(ra, rb, pr, G, stage, j); break;
    case Q8:  store_pair<Q8>(ra, rb, pr, G, stage, j);  break;
    default: break;
    }
}

// One operand of the same: piece i = 2 * (row block) + (0: A, 1: B).
__device__ __forceinline__ void load_piece(Raw &r, const Product &pr, int nb, int c, int i)
{
    const int eoff = c * chunk_elems(pr.q) + (i >> 1) * 32 * nb;
    const Operand &o = (i & 1) ? pr.b : pr.a;
    load_seg(r, o, eoff << (3 - o.p), pr.q == Q32 && o.p == Q64);
}
// The same without control flow, for a product known only at run time: the second half is
// always requested, through a descriptor of length zero (such a load touches no memory and
// returns zeros) unless the piece is the one down-cast.
__device__ __forceinline__ void load_piece_any(Raw &r, const Product &pr, int nb, int c, int i)
{
    const int eoff = c * chunk_elems(pr.q) + (i >> 1) * 32 * nb;
    const Operand &o = (i & 1) ? pr.b : pr.a;
    const bool down = pr.q == Q32 && o.p == Q64;
    const int soff = eoff << (3 - o.p);
    const __amdgpu_buffer_rsrc_t lo = __builtin_amdgcn_make_buffer_rsrc((void *)o.base, 0, o.bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t hi = __builtin_amdgcn_make_buffer_rsrc((void *)o.base, 0, down ? o.bytes : 0, 0x00020000);
    r.lo = __builtin_amdgcn_raw_buffer_load_b128(lo, o.voff, soff, 0);
    r.hi = __builtin_amdgcn_raw_buffer_load_b128(hi, o.voff + 16, soff, 0);
}
// The same where no piece is a down-cast (no FP64 tile under an FP32 product): the first half only.
__device__ __forceinline__ void load_piece_lo(Raw &r, const Product &pr, int nb, int c, int i)
{
    const int eoff = c * chunk_elems(pr.q) + (i >> 1) * 32 * nb;
    const Operand &o = (i & 1) ? pr.b : pr.a;
    const __amdgpu_buffer_rsrc_t lo = __builtin_amdgcn_make_buffer_rsrc((void *)o.base, 0, o.bytes, 0x00020000);
    r.lo = __builtin_amdgcn_raw_buffer_load_b128(lo, o.voff, eoff << (3 - o.p), 0);
    r.hi = u32x4{0, 0, 0, 0};                          // never read: only a down-cast looks at it
}
template <int Q>
__device__ __forceinline__ void store_piece(const Raw &r, const Product &pr, const Geometry &G, char *stage, int i)
{
    static_assert(Q == Q64 || Q == Q32, "swizzled stages only");
    const Operand &o = (i & 1) ? pr.b : pr.a;
    char *dst = stage + G.wsw + (i >> 1) * (32 * kRowBytes) + (i & 1) * kOperandStage;
    *(u32x4 *)dst = convert<Q>(r, o.p, o.e, o.sub);
}
__device__ __forceinline__ void store_piece_any(const Raw &r, const Product &pr, const Geometry &G, char *stage, int i)
{
    const Operand &o = (i & 1) ? pr.b : pr.a;
    switch (pr.q) {
    case Q64: store_piece<Q64>(r, pr, G, stage, i); break;
    case Q32: store_piece<Q32>(r, pr, G, stage, i); break;
    case Q16: lds_store16(stage + G.wbase + (i >> 1) * (32 * kRowStride) + (i & 1) * kOperandStage, convert<Q16>(r, o.p, o.e, o.sub)); break;
    case Q8:  lds_store16(stage + G.wbase + (i >> 1) * (32 * kRowStride) + (i & 1) * kOperandStage, convert<Q8>(r, o.p, o.e, o.sub)); break;
    default: break;
    }
}

// ---- staging with both stored precisions known at compile time (the steady chunks) -----------
// The generic staging above fetches the aligned 16 bytes around a segment's source and picks the
// source out of them at conversion time with per-lane selects, then converts and scales with
// one instruction each per element: vector-ALU work that FP64 / FP32 MFMAs do not hide.  With
// the stored precision P a template parameter the source is fetched exactly (2, 4 or 8 bytes:
// no selects) and conversion and scaling are fused: v_fma_mix_f32 takes an FP16 half straight
// out of a packed register and multiplies it by 2^e in FP32, v_cvt_scalef32_pk_f32_fp8 turns
// two FP8 bytes into two scaled FP32 values.  Both were checked on the device against
// cvt + ldexp over every bit pattern and a range of scales: v_fma_mix_f32 agrees for every
// scale that is an FP32 number, subnormal ones included (one correct rounding, also into the
// subnormal range); v_cvt_scalef32 for scales 2^-126 and up.  Towards FP64 the FP32 intermediate
// must itself be exact, which narrows the range further.  A product with a tile exponent
// outside these ranges (tiles whose largest entry is below about 1e-26, in FP64 C tiles, or
// 1e-36) runs its chunks through the generic staging instead.
struct HiScale {
    float f;      // 2^e
};
__device__ __forceinline__ HiScale hi_scale(int e)
{
    HiScale h;
    h.f = __uint_as_float(e >= -126 ? (uint32_t)(e + 127) << 23 : 1u << ((e + 149) & 31));
    return h;
}
// May an operand stored at precision p with tile exponent e take the fused conversions to Q?
template <int Q>
__device__ __forceinline__ bool fused_ok(int p, int e)
{
    if (p < Q16) return true;                                  // FP64 / FP32 storage carries no scale
    if (Q == Q32) return p == Q16 ? (e >= -149 && e <= 127) : (e >= -126 && e <= 127);
    return p == Q16 ? (e >= -102 && e <= 111) : (e >= -117 && e <= 118);
}
// The source of a converted 16-byte segment of precision Q stored at precision P: 16 bytes when
// P = Q, 32 for the one down-cast, else 16 * size(P) / size(Q).  o.voff is the exact offset here.
template <int Q, int P>
__device__ __forceinline__ void load_exact(Raw &r, const Operand &o, int soff)
{
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)o.base, 0, o.bytes, 0x00020000);
    constexpr int kBytes = P < Q ? 32 : 16 >> (P - Q);
    if constexpr (kBytes >= 16) {
        r.lo = __builtin_amdgcn_raw_buffer_load_b128(rsrc, o.voff, soff, 0);
        if constexpr (kBytes == 32) r.hi = __builtin_amdgcn_raw_buffer_load_b128(rsrc, o.voff + 16, soff, 0);
    } else if constexpr (kBytes == 8) {
        const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rsrc, o.voff, soff, 0);
        r.lo.x = v.x; r.lo.y = v.y;
    } else if constexpr (kBytes == 4) {
        r.lo.x = __builtin_amdgcn_raw_buffer_load_b32(rsrc, o.voff, soff, 0);
    } else {
        r.lo.x = __builtin_amdgcn_raw_buffer_load_b16(rsrc, o.voff, soff, 0);
    }
}
template <int WHICH>
__device__ __forceinline__ float half_scaled(uint32_t w, float f)     // half WHICH of w, times f, in FP32
{
    float x;
#if defined(__HIP_DEVICE_COMPILE__)
    // the addend is -0 so that a negative zero stays one
    const float nz = __uint_as_float(0x80000000u);
    if constexpr (WHICH == 0) asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(x) : "v"(w), "s"(f), "v"(nz));
    else asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(x) : "v"(w), "s"(f), "v"(nz));
#else
    x = 0.0f; (void)w; (void)f;
#endif
    return x;
}
template <int Q, int P>
__device__ __forceinline__ u32x4 convert_exact(const Raw &r, const HiScale &S)
{
    static_assert(Q == Q64 || Q == Q32, "FP64 / FP32 products only");
    if constexpr (P == Q) {
        return r.lo;
    } else if constexpr (Q == Q32 && P == Q64) {
        return u32x4{__float_as_uint((float)as_double(r.lo.x, r.lo.y)), __float_as_uint((float)as_double(r.lo.z, r.lo.w)),
                     __float_as_uint((float)as_double(r.hi.x, r.hi.y)), __float_as_uint((float)as_double(r.hi.z, r.hi.w))};
    } else if constexpr (Q == Q32) {
        float f0, f1, f2, f3;
        if constexpr (P == Q16) {
            f0 = half_scaled<0>(r.lo.x, S.f); f1 = half_scaled<1>(r.lo.x, S.f);
            f2 = half_scaled<0>(r.lo.y, S.f); f3 = half_scaled<1>(r.lo.y, S.f);
        } else {
            const f2v a = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(r.lo.x, S.f, false);
            const f2v b = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(r.lo.x, S.f, true);
            f0 = a.x; f1 = a.y; f2 = b.x; f3 = b.y;
        }
        return u32x4{__float_as_uint(f0), __float_as_uint(f1), __float_as_uint(f2), __float_as_uint(f3)};
    } else {
        double a, b;
        if constexpr (P == Q32) {
            a = (double)__uint_as_float(r.lo.x); b = (double)__uint_as_float(r.lo.y);
        } else {
            float f0, f1;
            if constexpr (P == Q16) {
                f0 = half_scaled<0>(r.lo.x, S.f); f1 = half_scaled<1>(r.lo.x, S.f);
            } else {
                const f2v v = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(r.lo.x, S.f, false);
                f0 = v.x; f1 = v.y;
            }
            a = (double)f0; b = (double)f1;
        }
        const u32x2 ab = dbits(a), bb = dbits(b);
        return u32x4{ab.x, ab.y, bb.x, bb.y};
    }
}
// Piece i = 2 * (row block) + (0: A, 1: B) of chunk c with the stored precisions PA, PB.
template <int Q, int PA, int PB>
__device__ __forceinline__ void load_piece_exact(Raw &r, const Product &pr, int nb, int c, int i)
{
    const int eoff = c * chunk_elems(Q) + (i >> 1) * 32 * nb;
    if (i & 1) load_exact<Q, PB>(r, pr.b, eoff << (3 - PB));
    else load_exact<Q, PA>(r, pr.a, eoff << (3 - PA));
}
template <int Q, int PA, int PB>
__device__ __forceinline__ void store_piece_exact(const Raw &r, const HiScale &SA, const HiScale &SB, const Geometry &G, char *stage, int i)
{
    char *dst = stage + G.wsw + (i >> 1) * (32 * kRowBytes) + (i & 1) * kOperandStage;
    if (i & 1) *(u32x4 *)dst = convert_exact<Q, PB>(r, SB);
    else *(u32x4 *)dst = convert_exact<Q, PA>(r, SA);
}

// Everything that describes a tile product is the same for all lanes of the workgroup; passing
// it through readfirstlane keeps it in scalar registers and makes every branch on it scalar.
// Wave-uniform reads of the small descriptor tables (read-only for the whole kernel) through
// the constant address space, so that they are scalar loads: no vector registers, no vector
// ALU, and no interference with the counter of outstanding vector-memory operations.  Byte
// tables are read as the aligned 32-bit word around the byte (the tables are allocated with
// padding).
typedef const __attribute__((address_space(4))) uint32_t *ConstWord;
typedef const __attribute__((address_space(4))) uint64_t *ConstDword;
__device__ __forceinline__ int table_i32(const int32_t *t, int64_t i) { return (int)*(ConstWord)(uintptr_t)(t + i); }
__device__ __forceinline__ uint64_t table_u64(const uint64_t *t, int64_t i) { return *(ConstDword)(uintptr_t)(t + i); }
__device__ __forceinline__ int table_u8(const uint8_t *t, int64_t i)
{
    const uintptr_t a = (uintptr_t)(t + i);
    return (int)((*(ConstWord)(a & ~(uintptr_t)3) >> ((a & 3) * 8)) & 0xffu);
}
// The kernel's arguments, read where they are needed from the kernel-argument segment (constant
// memory, scalar loads) instead of being held in scalar registers for the kernel's lifetime:
// there are some forty of them and the chunk loops need the registers.  The pointer is made
// opaque each time so that the reads are issued at the point of use.
typedef const __attribute__((address_space(4))) GemmArgs *ArgsPtr;
__device__ __forceinline__ ArgsPtr args()
{
#if defined(__HIP_DEVICE_COMPILE__)
    uint64_t p = (uint64_t)__builtin_amdgcn_kernarg_segment_ptr();
    asm volatile("" : "+s"(p));
    return (ArgsPtr)p;
#else
    return (ArgsPtr)0;
#endif
}

__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ const char *uni(const char *p)
{
    const uint64_t v = (uint64_t)p;
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
    return (const char *)(((uint64_t)hi << 32) | lo);
}

// Descriptor of one operand tile from its table entries; `row0` is the first tile row this
// workgroup reads.
__device__ __forceinline__ Operand make_operand(const char *base, int p, int e, int q, int row0, const Geometry &G, int nb, int fmt)
{
    Operand o;
    o.base = base;
    o.p = p;
    o.e = e;
    const int shift = 3 - o.p;                                   // log2 of the element size
    const int n_q = 2 << q;                                      // elements per 16-byte converted segment
    const int eidx = (row0 + G.seg_row) * nb + G.seg_part * n_q; // this thread's first element
    const int elems = fmt == 3 ? (nb * nb) >> 1 : (nb * nb) << shift;   // bytes of the tile's elements (MXFP4: two to a byte)
    o.bytes = fmt >= 2 ? elems + ((nb * nb) >> 5) : elems;       // block-scaled: one scale byte per 32 elements behind them
    const int boff = fmt == 3 ? eidx >> 1 : eidx << shift;
    o.voff = boff & ~15;
    o.sub = (boff & 15) | (fmt << 8);
    return o;
}

// Load the descriptors of tile product L of this C tile (q = -1 past the end): one 32-byte
// scalar load from the product table.
typedef const __attribute__((address_space(4))) u32x4 *ConstQuad;
__device__ __forceinline__ Product make_product(const u32x4 lo, const u32x4 hi, const Geometry &G, const Region &R)
{
    Product pr;
    const uint64_t pta = (uint64_t)lo.x | ((uint64_t)lo.y << 32), ptb = (uint64_t)lo.z | ((uint64_t)lo.w << 32);
    const int ea = (int)hi.x, eb = (int)hi.y;
    const int ca = (int)(hi.z & 0xffu), cb = (int)((hi.z >> 8) & 0xffu), q = (int)((hi.z >> 16) & 0xffu);
    // bits 24 / 25: the A / B tile holds BF16 numbers (written as FP16 in the codes: the same element
    // size); codes 5 / 6 / 7: an MXFP8 / MXFP4 / MXFP6 tile under an FP32 / FP64 product, read like an
    // FP8 tile whose scale comes per block
    const int fa = ca >= GEMM_MP_MXFP8 ? ca - GEMM_MP_MXFP8 + 2 : (int)((hi.z >> 24) & 1u);
    const int fb = cb >= GEMM_MP_MXFP8 ? cb - GEMM_MP_MXFP8 + 2 : (int)((hi.z >> 25) & 1u);
    const int pa = ca >= GEMM_MP_MXFP8 ? (int)Q8 : ca, pb = cb >= GEMM_MP_MXFP8 ? (int)Q8 : cb;
    pr.q = q;
    pr.a = make_operand((const char *)(uintptr_t)pta, pa, ea, q, R.arow0, G, R.nb, fa);
    pr.b = make_operand((const char *)(uintptr_t)ptb, pb, eb, q, R.brow0, G, R.nb, fb);
    return pr;
}
__device__ __forceinline__ Product open_product(int I, int J, int tileC, int L, const Geometry &G, const Region &R)
{
    (void)I; (void)J; (void)tileC;
    Product pr;
    pr.q = -1;
    pr.a = Operand{};
    pr.b = Operand{};
    if (L >= R.kt_eff) return pr;
    const ConstQuad rec = (ConstQuad)(uintptr_t)(R.prod + L);
    const u32x4 lo = rec[0], hi = rec[1];
    return make_product(lo, hi, G, R);
}

// What a product loop needs in order to open the following tile product itself.
struct Walk {
    int I, J, tileC;
};

// Per-lane LDS offsets of the fragment rows in a padded stage (stage 0): A rows of this wave's
// 64 x 64 part and B rows; row block t adds t * 16 * kRowStride, 8 w bytes select the word.
struct FragBase {
    const char *a, *b;
};
template <int Q>
__device__ __forceinline__ FragBase frag_base(const char *lds, const Geometry &G)
{
    FragBase f;
    f.a = lds + (G.wm * 64 + G.li) * kRowStride + G.g * 32;
    f.b = lds + kOperandStage + (G.wn * 64 + G.li) * kRowStride + G.g * 32;
    return f;
}
// The same for a swizzled stage.  Lane (li, g) reads the two 16-byte segments 2g and 2g + 1 of
// its row (macro-steps 0 and 1 of a chunk): element h of segment 2g + j is reduction index
// (2g + j) * n + h of the chunk (n = 2 FP64 or 4 FP32 elements per segment) in A and B alike,
// so each k-step's MFMA pairs equal indices; the order in which a chunk's indices are summed
// is a permutation of the storage order.  Row block t adds t * 16 * kRowBytes.
struct HiFrag {
    const char *a[2], *b[2];
};
template <int Q>
__device__ __forceinline__ HiFrag hi_frag(const char *lds, const Geometry &G)
{
    // FP64 accumulators hold C[4v+g][i] where the FP32-result ones hold C[4g+v][i]; reading A row
    // 4*(i%4) + i/4 in lane i on the FP64 path makes both address the same C element.
    const int arow = (Q == Q64) ? 4 * (G.li & 3) + (G.li >> 2) : G.li;
    const int sa = (2 * G.g) ^ ((arow >> 1) & 7), sb = (2 * G.g) ^ ((G.li >> 1) & 7);
    HiFrag f;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        f.a[j] = lds + (G.wm * 64 + arow) * kRowBytes + ((sa ^ j) * 16);
        f.b[j] = lds + kOperandStage + (G.wn * 64 + G.li) * kRowBytes + ((sb ^ j) * 16);
    }
    return f;
}
__device__ __forceinline__ u32x4 lds_load16(const char *p) { return *(const u32x4 *)p; }
__device__ __forceinline__ u32x2 lds_load8(const char *p) { return *(const u32x2 *)p; }

// The FP32 accumulators of the FP64 / FP32 product loops live in fixed registers: accumulator
// (mt, nt) of the pinned set is v[192 + 4 (4 mt + nt) : + 3].  Left to the register allocator,
// every specialised loop gets its own assignment, with register-to-register copies on the way
// in and out of each tile product's loop (pinning measured 0.5-1.5 % on FP32 tiles).  They are
// vector registers, not accumulation registers (an MFMA takes either): the folds and the
// epilogue, which are vector-ALU code, then work on them in place.
// BASE: 192 = the pinned set (the running sum of an FP32 C tile), -1 = wherever the allocator
// puts them (accumulation registers: the per-product accumulator of an FP64 C tile, whose
// kernel has no vector registers to spare).
#define GMP_VQUADS(X) X(192, 192, 195) X(196, 196, 199) X(200, 200, 203) X(204, 204, 207) X(208, 208, 211) X(212, 212, 215) X(216, 216, 219) X(220, 220, 223) X(224, 224, 227) X(228, 228, 231) X(232, 232, 235) X(236, 236, 239) X(240, 240, 243) X(244, 244, 247) X(248, 248, 251) X(252, 252, 255)
template <int R>
__device__ __forceinline__ void mfma_f32_at(f4 &acc, uint32_t a, uint32_t b)
{
#define X(R0, LO, HI) if constexpr (R == R0) asm volatile("v_mfma_f32_16x16x4_f32 %0, %1, %2, %0" : "+{v[" #LO ":" #HI "]}"(acc) : "v"(a), "v"(b));
    GMP_VQUADS(X)
#undef X
    if constexpr (R < 0) asm volatile("v_mfma_f32_16x16x4_f32 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}

// ---- FP64 / FP32 products: software-pipelined chunk loop -----------------------------------
// A chunk is two macro-steps of 16 bytes of reduction index per lane: two FP64 k-steps (32 MFMAs
// of 64 cycles) or four FP32 k-steps (64 MFMAs of 32 cycles) each.  FP64 / FP32 MFMAs do not
// overlap with vector-ALU instructions, and memory instructions issued in a burst stall the
// MFMA stream far longer than the same instructions issued one at a time (measured: four LDS
// writes back to back cost 140 cycles, one between MFMAs about 4).  The chunk is therefore a
// sequence of 64 positions, one after every FP64 MFMA or every second FP32 MFMA, and each
// position holds at most one other instruction:
//   positions  0..15 : global loads of the next chunk (even) and LDS reads of macro-step 1's
//                      fragments (odd)
//   positions 34..48 : conversion + LDS write of the next chunk into the other stage (even)
//   position  52     : barrier
//   positions 53..60 : LDS reads of the next chunk's first fragments
// fr[buf][0..3] = A fragments of row blocks 0..3, fr[buf][4..7] = B fragments.
// The FP32 MFMAs are written as asm so that the accumulator is read and written in place in an
// accumulation register: left to itself the register allocator rotates the FP32 side
// accumulators through other registers with a copy per loop iteration.  Asm MFMAs are invisible
// to the compiler's hazard handling, so the first one of a chunk carries wait states in front (a
// register copy or zeroing may sit right before it) and the last one carries the wait states an
// 8-pass MFMA needs before an ordinary instruction may touch its result.
// Half-quad u = 0..63 of a chunk: FP32: (macro-step j, row block mt, element h, columns nt0,
// nt0 + 1); FP64: one MFMA.
template <int Q, int BASE, int u, typename Acc>
__device__ __forceinline__ void mfma_half(Acc (&acc)[4][4], const u32x4 (&fr)[2][8])
{
    constexpr int j = u >> 5, mt = (u >> 3) & 3;
    if constexpr (Q == Q64) {
        constexpr int h = (u >> 2) & 1, nt = u & 3;
        acc[mt][nt] = __builtin_amdgcn_mfma_f64_16x16x4f64(as_double(fr[j][mt][2 * h], fr[j][mt][2 * h + 1]),
                                                           as_double(fr[j][4 + nt][2 * h], fr[j][4 + nt][2 * h + 1]), acc[mt][nt], 0, 0, 0);
    } else {
        constexpr int h = (u >> 1) & 3, nt0 = (u & 1) * 2;
        if constexpr (u == 0) asm volatile("s_nop 3");
        mfma_f32_at<(BASE < 0 ? -1 : BASE + 4 * (4 * mt + nt0))>(acc[mt][nt0], fr[j][mt][h], fr[j][4 + nt0][h]);
        mfma_f32_at<(BASE < 0 ? -1 : BASE + 4 * (4 * mt + nt0 + 1))>(acc[mt][nt0 + 1], fr[j][mt][h], fr[j][4 + nt0 + 1][h]);
        if constexpr (u == 63) asm volatile("s_nop 11");
    }
}

// The asm MFMAs are invisible to the compiler's hazard handling.  Around every run of them a
// fence takes all sixteen accumulators as in/out accumulation registers and waits 32 cycles:
// whatever register copies the compiler needs are placed outside the fenced region, after the
// last MFMA has retired and long enough before the first one issues.
template <int BASE, typename Acc>
__device__ __forceinline__ void acc_fence(Acc (&acc)[4][4])
{
    if constexpr (std::is_same<Acc, f4>::value) {
        if constexpr (BASE < 0)
            asm volatile("s_nop 15\n\ts_nop 15"
                         : "+a"(acc[0][0]), "+a"(acc[0][1]), "+a"(acc[0][2]), "+a"(acc[0][3]),
                           "+a"(acc[1][0]), "+a"(acc[1][1]), "+a"(acc[1][2]), "+a"(acc[1][3]),
                           "+a"(acc[2][0]), "+a"(acc[2][1]), "+a"(acc[2][2]), "+a"(acc[2][3]),
                           "+a"(acc[3][0]), "+a"(acc[3][1]), "+a"(acc[3][2]), "+a"(acc[3][3]));
        if constexpr (BASE == 192) asm volatile("s_nop 15\n\ts_nop 15" : "+{v[192:195]}"(acc[0][0]), "+{v[196:199]}"(acc[0][1]), "+{v[200:203]}"(acc[0][2]), "+{v[204:207]}"(acc[0][3]), "+{v[208:211]}"(acc[1][0]), "+{v[212:215]}"(acc[1][1]), "+{v[216:219]}"(acc[1][2]), "+{v[220:223]}"(acc[1][3]), "+{v[224:227]}"(acc[2][0]), "+{v[228:231]}"(acc[2][1]), "+{v[232:235]}"(acc[2][2]), "+{v[236:239]}"(acc[2][3]), "+{v[240:243]}"(acc[3][0]), "+{v[244:247]}"(acc[3][1]), "+{v[248:251]}"(acc[3][2]), "+{v[252:255]}"(acc[3][3]));
    }
}

// Fragment t (0..3: A row blocks, 4..7: B row blocks) of macro-step j from the stage at byte
// offset `so`.
__device__ __forceinline__ u32x4 read_frag(const HiFrag &F, int so, int j, int t)
{
    constexpr int kBlock = 16 * kRowBytes;
    return t < 4 ? lds_load16(F.a[j] + so + t * kBlock) : lds_load16(F.b[j] + so + (t - 4) * kBlock);
}

// One position of a chunk: MFMAs, then at most one other instruction.
// pr / c: product and chunk index of the chunk to fetch: the next chunk of this product, or,
// when LAST, chunk 0 of the next product, which is only loaded into `r`: its conversion is
// specialised on that product's stored precisions and therefore left to that product's loop.
struct ChunkCtx {
    int so, no;        // byte offsets of the stage computed from and of the one being filled
    char *wst;         // the latter's address
    HiScale sa, sb;    // MODE 0: the operands' scales
};
// MODE: 3 = as 2 where no operand is an FP64 tile under an FP32 product: only the first 16 bytes
// of a piece are fetched, and only they stay in registers until the next product's loop.
// MODE: 0 = a chunk followed by another of the same product; 1 = the last chunk, which also
// stages chunk 0 of the next product (conversion chosen at run time); 2 = the last chunk, which
// only loads it into `r` (the next product's own loop converts and stores it).
template <int Q, int BASE, int MODE, int PA, int PB, int u, typename Acc>
__device__ __forceinline__ void chunk_position(Acc (&acc)[4][4], u32x4 (&fr)[2][8], Raw (&r)[8], const Product &pr, int c, const ChunkCtx &X,
                                               const HiFrag &F, const Geometry &G, int nb)
{
    mfma_half<Q, BASE, u>(acc, fr);
    SCHED_FENCE();
    if constexpr (u < 16 && (u & 1) == 0) {
        if constexpr (MODE == 3) load_piece_lo(r[u >> 1], pr, nb, c, u >> 1);
        else if constexpr (MODE != 0) load_piece_any(r[u >> 1], pr, nb, c, u >> 1);
        else if constexpr (PA >= 0) load_piece_exact<Q, PA, PB>(r[u >> 1], pr, nb, c, u >> 1);
        else load_piece(r[u >> 1], pr, nb, c, u >> 1);
    } else if constexpr (u < 16) {
        constexpr int t = ((u >> 1) + 4) & 7;                // B0..B3, A0..A3
        fr[1][t] = read_frag(F, X.so, 1, t);
    } else if constexpr (MODE != 2 && MODE != 3 && u >= 34 && u <= 48 && (u & 1) == 0) {
        constexpr int i = (u - 34) >> 1;
        if constexpr (MODE == 0 && PA >= 0) store_piece_exact<Q, PA, PB>(r[i], X.sa, X.sb, G, X.wst, i);
        else if constexpr (MODE == 0) store_piece<Q>(r[i], pr, G, X.wst, i);
        else store_piece_any(r[i], pr, G, X.wst, i);   // q < 0 (nothing follows): stores nothing
    } else if constexpr (MODE != 2 && MODE != 3 && u == 52) {
        __syncthreads();
    } else if constexpr (MODE == 0 && u >= 53 && u <= 60) {
        constexpr int t = (u - 53 + 4) & 7;                  // B0..B3, A0..A3
        fr[0][t] = read_frag(F, X.no, 0, t);
    }
    SCHED_FENCE();
}
template <int Q, int BASE, int MODE, int PA, int PB, typename Acc, int... U>
__device__ __forceinline__ void chunk_positions(Acc (&acc)[4][4], u32x4 (&fr)[2][8], Raw (&r)[8], const Product &pr, int c, const ChunkCtx &X,
                                                const HiFrag &F, const Geometry &G, int nb, std::integer_sequence<int, U...>)
{
    (chunk_position<Q, BASE, MODE, PA, PB, U>(acc, fr, r, pr, c, X, F, G, nb), ...);
}
// STAGE: the LDS stage the chunk computes from when it is known at compile time (0 / 1; the
// stage offsets then fold into the instructions' immediate offsets instead of costing vector
// adds every chunk), -1: taken from `stage`.
template <int Q, int BASE, int MODE, int STAGE = -1, int PA = -1, int PB = -1, typename Acc>
__device__ __forceinline__ void pipelined_chunk(Acc (&acc)[4][4], u32x4 (&fr)[2][8], Raw (&r)[8], const Product &pr, int c, char *lds, int stage,
                                                const HiFrag &F, const Geometry &G, int nb, const HiScale &sa = HiScale{}, const HiScale &sb = HiScale{})
{
    if (STAGE >= 0) stage = STAGE;
    ChunkCtx X;
    X.sa = sa;
    X.sb = sb;
    X.so = stage * kStage;
    X.no = (stage ^ 1) * kStage;
    X.wst = lds + X.no;
    chunk_positions<Q, BASE, MODE, PA, PB>(acc, fr, r, pr, c, X, F, G, nb, std::make_integer_sequence<int, 64>{});
}

// All but the last chunk of a product whose operands are stored at precisions PA, PB: with
// both known at compile time the staging code is straight-line (no conversion at all when
// PA = PB = Q).  PA = PB = -1: any precisions, any exponents, conversion chosen at run time.  On entry the product's chunk 0 is either staged in LDS stage `stage` or, when
// `raw`, still in `hand` as loaded by the preceding product's last chunk.
template <int Q, int BASE, int PA, int PB, typename Acc>
__device__ __forceinline__ void steady_chunks(Acc (&acc)[4][4], u32x4 (&fr)[2][8], const Product &cur, int n, char *lds, int &stage,
                                              const HiFrag &F, const Geometry &G, int nb, Raw (&hand)[8], bool raw)
{
    Product cp = cur;
    cp.q = Q;
    if constexpr (PA >= 0) {
        cp.a.p = PA;
        cp.b.p = PB;
    }
    if (raw) {
#pragma unroll
        for (int i = 0; i < 8; ++i) store_piece<Q>(hand[i], cp, G, lds + stage * kStage, i);
        __syncthreads();
    }
#pragma unroll
    for (int t = 4; t < 12; ++t) fr[0][t & 7] = read_frag(F, stage * kStage, 0, t & 7);
    acc_fence<BASE>(acc);
    Raw r[8];
    int c = 1;
    if constexpr (PA < 0) {
        // operands at any stored precision with any exponent: conversion chosen at run time
        for (; c < n; ++c) {
            pipelined_chunk<Q, BASE, 0>(acc, fr, r, cp, c, lds, stage, F, G, nb);
            stage ^= 1;
        }
        return;
    }
    const HiScale sa = hi_scale(cp.a.e), sb = hi_scale(cp.b.e);
    // from here on the operands' vector offsets are exact (the generic staging keeps them
    // aligned down to 16 bytes with the remainder in `sub`)
    cp.a.voff += cp.a.sub;
    cp.b.voff += cp.b.sub;
    // Chunks run in pairs with the LDS stage a compile-time constant: the stage offsets fold into
    // the instructions' immediate fields instead of costing vector adds in every chunk (+2 to
    // +4 % on every operand mix).
    if (stage == 1 && c < n) {                         // bring the loop to stage 0
        pipelined_chunk<Q, BASE, 0, 1, PA, PB>(acc, fr, r, cp, c, lds, 1, F, G, nb, sa, sb);
        stage = 0;
        ++c;
    }
    for (; c + 1 < n; c += 2) {                        // pairs of chunks with the stages known
        pipelined_chunk<Q, BASE, 0, 0, PA, PB>(acc, fr, r, cp, c, lds, 0, F, G, nb, sa, sb);
        pipelined_chunk<Q, BASE, 0, 1, PA, PB>(acc, fr, r, cp, c + 1, lds, 1, F, G, nb, sa, sb);
    }
    if (c < n) {
        pipelined_chunk<Q, BASE, 0, 0, PA, PB>(acc, fr, r, cp, c, lds, 0, F, G, nb, sa, sb);
        stage = 1;
    }
}

// ---- FP64 / FP32 products with a BF16, MXFP8, MXFP4 or MXFP6 operand ---------------------------------
// Receiver-side conversion of the formats beyond the paper's: a BF16 number is the upper half of
// an FP32 word, a block-scaled element times the scale 2^(code - 127) of its block of 32 is exact
// in FP32 (and FP64).  These products take a plain loop of their own: per chunk, fetch the eight
// pieces (and, for a block-scaled tile, the scale byte of each segment's block: the blocks run
// along the rows of the packed tile, one byte each, row by row behind the elements), convert, store
// to LDS stage 0, and run the chunk's matrix instructions; nothing is overlapped.  The fast roads
// for such tiles are their own kernels (BF16 x BF16, MXFP8 x MXFP8, MXFP4 x MXFP4 products) and
// sender-side copies; this one keeps every tile convertible by its consumer.
// Number of a narrow code (sign, two exponent bits with bias 1, mb fraction bits: e2m1 with mb = 1,
// e2m3 with mb = 3) times 2^e; exact in FP32.
__device__ __forceinline__ float narrow_value(uint32_t code, int mb, int e)
{
    const int mf = (int)code & ((1 << mb) - 1), ef = (int)(code >> mb) & 3;
    const int mant = ef ? ((1 << mb) + mf) << (ef - 1) : mf;   // in units of 2^-mb
    const float mag = ldexpf((float)mant, e - mb);
    return ((code >> (mb + 2)) & 1u) ? -mag : mag;
}
// Piece i = 2 * (row block) + (0: A, 1: B) of chunk c: the aligned 16 bytes around the source, the
// second 16 for the one down-cast, the scale byte (into r.hi.x) for a block-scaled tile.
__device__ __forceinline__ void load_piece_widening(Raw &r, const Product &pr, int nb, int c, int i)
{
    const int eoff = c * chunk_elems(pr.q) + (i >> 1) * 32 * nb;
    const Operand &o = (i & 1) ? pr.b : pr.a;
    const int fmt = __builtin_amdgcn_readfirstlane(o.sub >> 8);
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)o.base, 0, o.bytes, 0x00020000);
    if (fmt >= 3) {
        // MXFP4 / MXFP6: W = 4 / 6 bits per element.  The operand's descriptor counts in bytes of
        // an element size the kernel knows (MXFP4: two elements a byte; MXFP6 is announced like
        // MXFP8, one byte per element), which gives back the thread's first element.  The two
        // aligned words around its codes are read (at most 24 bits from bit 28 of the first), and
        // the bit offset in them goes along in r.hi.y.  MXFP4 codes lie row after row; where the
        // three bytes of four MXFP6 codes lie is fp6_group_offset's business.
        const int e0 = ((o.voff + (o.sub & 15)) << (fmt == 3 ? 1 : 0)) + eoff;
        int byte, bit;
        if (fmt == 3) {
            byte = e0 >> 1;
            bit = 8 * (byte & 3);
        } else {
            const int row = e0 / nb, k = e0 - row * nb;
            byte = (int)fp6_group_offset(nb, row, k & ~3);
            bit = 8 * (byte & 3) + 6 * (k & 3);
        }
        const u32x2 w = __builtin_amdgcn_raw_buffer_load_b64(rsrc, byte & ~3, 0, 0);
        r.lo.x = w.x;
        r.lo.y = w.y;
        r.hi.y = (uint32_t)bit;
        r.hi.x = (uint32_t)__builtin_amdgcn_raw_buffer_load_b8(rsrc, ((nb * nb * (fmt == 3 ? 4 : 6)) >> 3) + (e0 >> 5), 0, 0);
        return;
    }
    r.lo = __builtin_amdgcn_raw_buffer_load_b128(rsrc, o.voff, eoff << (3 - o.p), 0);
    if (pr.q == Q32 && o.p == Q64) {
        r.hi = __builtin_amdgcn_raw_buffer_load_b128(rsrc, o.voff + 16, eoff << (3 - o.p), 0);
    } else if (fmt == 2) {
        // the element index comes back from the byte offset of the segment's source
        const int boff = o.voff + (o.sub & 15);
        r.hi.x = (uint32_t)__builtin_amdgcn_raw_buffer_load_b8(rsrc, nb * nb + (boff >> 5), eoff >> 5, 0);
    }
}
template <int Q>
__device__ __forceinline__ u32x4 convert_widening(const Raw &r, const Operand &op)
{
    static_assert(Q == Q64 || Q == Q32, "FP64 / FP32 products only");
    const int fmt = __builtin_amdgcn_readfirstlane(op.sub >> 8), sub = op.sub & 15;
    if (fmt == 0) return convert<Q>(r, op.p, op.e, sub);
    u32x4 o;
    if (fmt == 1) {                                              // BF16: no scale
        if constexpr (Q == Q32) {
            const u32x2 w = pick_pair(r.lo, sub >> 3);
            o = u32x4{w.x << 16, w.x & 0xffff0000u, w.y << 16, w.y & 0xffff0000u};
        } else {
            const uint32_t w = pick_word(r.lo, sub >> 2);
            const u32x2 a = dbits((double)__uint_as_float(w << 16)), b = dbits((double)__uint_as_float(w & 0xffff0000u));
            o = u32x4{a.x, a.y, b.x, b.y};
        }
        return o;
    }
    const int e = (int)(r.hi.x & 0xffu) - 127;                   // this segment's block scale
    if (fmt == 2) return convert<Q>(r, Q8, e, sub);              // e4m3 elements: the FP8 road with the block's exponent
    // MXFP4 / MXFP6: four (FP32) or two (FP64) codes of W bits from bit r.hi.y of the loaded eight bytes
    const int W = fmt == 3 ? 4 : 6, mb = W - 3;
    const uint64_t both = (uint64_t)r.lo.x | ((uint64_t)r.lo.y << 32);
    const uint32_t w = (uint32_t)(both >> r.hi.y);
    const uint32_t mask = (1u << W) - 1u;
    if constexpr (Q == Q32) {
        o = u32x4{__float_as_uint(narrow_value(w & mask, mb, e)), __float_as_uint(narrow_value((w >> W) & mask, mb, e)),
                  __float_as_uint(narrow_value((w >> (2 * W)) & mask, mb, e)), __float_as_uint(narrow_value((w >> (3 * W)) & mask, mb, e))};
    } else {
        const u32x2 a = dbits(ldexp((double)narrow_value(w & mask, mb, 0), e)), b = dbits(ldexp((double)narrow_value((w >> W) & mask, mb, 0), e));
        o = u32x4{a.x, a.y, b.x, b.y};
    }
    return o;
}
template <int Q, int BASE, typename Acc, int... U>
__device__ __forceinline__ void chunk_mfmas(Acc (&acc)[4][4], const u32x4 (&fr)[2][8], std::integer_sequence<int, U...>)
{
    (mfma_half<Q, BASE, U>(acc, fr), ...);
}
// All chunks of such a product; returns the next product, whose first chunk (if it wants one) is
// staged in LDS stage 0 on exit, as after a run of ring products.
template <int Q, int BASE, bool MIXED, typename Acc>
__device__ __forceinline__ Product product_loop_widening(Acc (&acc)[4][4], const Product &cur, const Walk &W, int Lnext, char *lds, int &stage,
                                                         const Geometry &G0, const Region &R, bool &raw)
{
    const Geometry G = fresh(G0);
    const HiFrag F = hi_frag<Q>(lds, G);
    const int n = R.nb / (kRowBytes >> (3 - Q));
    const Product next = open_product(W.I, W.J, W.tileC, Lnext, G, R);
    Product cp = cur;
    cp.q = Q;
#pragma unroll 1
    for (int c = 0; c < n; ++c) {
        Raw r[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) load_piece_widening(r[i], cp, R.nb, c, i);
        __syncthreads();                               // every wave has read the chunk before from the stage
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            char *dst = lds + G.wsw + (i >> 1) * (32 * kRowBytes) + (i & 1) * kOperandStage;
            *(u32x4 *)dst = convert_widening<Q>(r[i], (i & 1) ? cp.b : cp.a);
        }
        __syncthreads();
        u32x4 fr[2][8];
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            fr[0][t] = read_frag(F, 0, 0, t);
            fr[1][t] = read_frag(F, 0, 1, t);
        }
        acc_fence<BASE>(acc);
        chunk_mfmas<Q, BASE>(acc, fr, std::make_integer_sequence<int, 64>{});
        acc_fence<BASE>(acc);
    }
    __syncthreads();
    if (wants_first_chunk<MIXED>(next, G)) {
        Raw xa[4], xb[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) load_pair(xa[j], xb[j], next, R.nb, 0, j);
#pragma unroll
        for (int j = 0; j < 4; ++j) store_pair_any(xa[j], xb[j], next, G, lds, j);
        __syncthreads();
    }
    stage = 0;
    raw = false;
    return next;
}

// All chunks of one FP64 / FP32 tile product; returns the next product.  On exit that one's
// chunk 0 is in `hand` (raw = true: it is an FP64 / FP32 product too), or staged in LDS stage
// `stage` (any other product that wants it).
// LATE: 0 = the last chunk stages the next product's first chunk in LDS; 1 = it only loads it, and
// the next product's own loop converts and stores it; 2 = as 1 in a kernel without FP64 products
// (no FP64 tile feeds an FP32 product: half the registers on the way).
template <int Q, int BASE, int LATE, bool MIXED, typename Acc>
__device__ __forceinline__ Product product_loop_pipelined(Acc (&acc)[4][4], const Product &cur, const Walk &W, int Lnext, char *lds, int &stage,
                                                          const Geometry &G0, const Region &R, Raw (&hand)[8], bool &raw)
{
    const Geometry G = fresh(G0);
    const HiFrag F = hi_frag<Q>(lds, G);
    u32x4 fr[2][8];
    const int n = R.nb / (kRowBytes >> (3 - Q));
    // the following product's descriptors: read now, needed only at this product's last chunk
    const Product next = open_product(W.I, W.J, W.tileC, Lnext, G, R);
#define GMP_STEADY(PA, PB) case (PA) * 4 + (PB): steady_chunks<Q, BASE, PA, PB>(acc, fr, cur, n, lds, stage, F, G, R.nb, hand, raw); break;
    // a scaled operand (FP16 / FP8) whose tile exponent is outside the fused conversions' range
    const bool wide = !fused_ok<Q>(cur.a.p, cur.a.e) || !fused_ok<Q>(cur.b.p, cur.b.e);
    switch (wide ? 16 : cur.a.p * 4 + cur.b.p) {
    case 16: steady_chunks<Q, BASE, -1, -1>(acc, fr, cur, n, lds, stage, F, G, R.nb, hand, raw); break;
        GMP_STEADY(0, 0) GMP_STEADY(0, 1) GMP_STEADY(0, 2) GMP_STEADY(0, 3)
        GMP_STEADY(1, 0) GMP_STEADY(1, 1) GMP_STEADY(1, 2) GMP_STEADY(1, 3)
        GMP_STEADY(2, 0) GMP_STEADY(2, 1) GMP_STEADY(2, 2) GMP_STEADY(2, 3)
        GMP_STEADY(3, 0) GMP_STEADY(3, 1) GMP_STEADY(3, 2) GMP_STEADY(3, 3)
    default: break;
    }
#undef GMP_STEADY
    acc_fence<BASE>(acc);
    const bool want = wants_first_chunk<MIXED>(next, G);
    Product ld = next;                                 // nothing to fetch: descriptors of length zero
    ld.a.bytes = want ? next.a.bytes : 0;
    ld.b.bytes = want ? next.b.bytes : 0;
    if constexpr (LATE != 0) {
        pipelined_chunk<Q, BASE, (LATE == 2 ? 3 : 2)>(acc, fr, hand, ld, 0, lds, stage, F, G, R.nb);
        acc_fence<BASE>(acc);
        stage ^= 1;
        raw = want && next.q <= Q32;
        if (want && !raw) {                            // a product of the padded two-stage loop: staged here
#pragma unroll
            for (int i = 0; i < 8; ++i) store_piece_any(hand[i], next, G, lds + stage * kStage, i);
            __syncthreads();
        }
    } else {
        if (!want) ld.q = -1;
        pipelined_chunk<Q, BASE, 1>(acc, fr, hand, ld, 0, lds, stage, F, G, R.nb);
        acc_fence<BASE>(acc);
        stage ^= 1;
        raw = false;
    }
    return next;
}

// ---- FP16 / FP8 products --------------------------------------------------------------------
// These MFMAs are fast (a chunk is ~530 matrix-core cycles per wave) and, unlike the FP64/FP32
// ones, overlap with vector-ALU work; what limits them is the latency of global memory and the
// LDS.  Consecutive FP16/FP8 products of a C region are therefore run as one stream of chunks
// through a ring of five LDS stages, each chunk requested four chunks ahead.  An operand
// stored in the product's own precision goes from global memory straight into LDS with the
// buffer-load-to-LDS instruction (no registers, no vector ALU).  An FP8 tile feeding an FP16
// product travels the same way, as FP8: its chunk rows are 64 bytes (the same 64 reduction
// indices), a DMA instruction covers 16 of them, so two of a wave's four instructions per
// operand carry data and the other two are empty; row r of the chunk lies at
// (r / 32) * 4096 + (r % 32) * 64 of the operand's stage.  A lane's fragments of both k-steps
// are then one 16-byte read (segment g of the row), converted to FP16 in registers, exactly
// (every e4m3 number is a binary16 number), in the shadow of the MFMAs.
struct LoGeom {
    int dma_row;      // tile row this lane fetches in DMA instruction j = 0 of its wave (+ 8 j)
    int dma_seg;      // byte offset of its 16-byte segment in the 128-byte chunk row
    int wbase;        // register path: swizzled LDS offset of (seg_row, seg_part); + 4096 j
    int fa0, fa1;     // fragment reads, A rows of this wave, row block 0: the lane's two 16-byte halves
    int fb0, fb1;     // same for B (includes the operand offset)
};
struct MixGeom {      // FP8 operand of an FP16 product
    int row;          // tile row this lane fetches in DMA instruction j = 0 of its wave (+ 16 j) ...
    int seg;          // ... and the byte offset of its 16-byte segment in the 64-byte chunk row
    int ma, mb;       // fragment reads: the lane's 16 bytes of row block 0 of A / of B
};

__device__ __forceinline__ LoGeom lo_geometry(const Geometry &G)
{
    LoGeom g;
    const int wave = G.tid >> 6;
    g.dma_row = wave * 32 + (G.lane >> 3);
    g.dma_seg = ((G.lane & 7) ^ ((G.lane >> 3) & 7)) * 16;
    g.wbase = G.seg_row * kRowBytes + ((G.seg_part ^ (G.seg_row & 7)) * 16);
    const int x = G.li & 7;
    g.fa0 = (G.wm * 64 + G.li) * kRowBytes + (((2 * G.g) ^ x) * 16);
    g.fa1 = (G.wm * 64 + G.li) * kRowBytes + (((2 * G.g + 1) ^ x) * 16);
    g.fb0 = kLoOperand + (G.wn * 64 + G.li) * kRowBytes + (((2 * G.g) ^ x) * 16);
    g.fb1 = kLoOperand + (G.wn * 64 + G.li) * kRowBytes + (((2 * G.g + 1) ^ x) * 16);
    return g;
}

__device__ __forceinline__ MixGeom mix_geometry(const Geometry &G)
{
    MixGeom g;
    g.row = (G.tid >> 6) * 32 + (G.lane >> 2);
    g.seg = (G.lane & 3) * 16;
    g.ma = G.wm * 8192 + G.li * 64 + G.g * 16;
    g.mb = kLoOperand + G.wn * 8192 + G.li * 64 + G.g * 16;
    return g;
}

typedef int i32x4 __attribute__((ext_vector_type(4)));

// Wait until at most `newer` vector-memory operations are outstanding.  Loads complete in
// order, so this guarantees the ones issued before the newest `newer` have landed; operations
// the compiler issued on its own in between only make the wait stricter.
__device__ __forceinline__ void lo_wait_dma(int newer)
{
#if defined(__HIP_DEVICE_COMPILE__)
    if (newer >= 24) asm volatile("s_waitcnt vmcnt(24)" ::: "memory");
    else if (newer >= 16) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
    else if (newer >= 12) asm volatile("s_waitcnt vmcnt(12)" ::: "memory");
    else if (newer >= 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    else if (newer >= 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#else
    (void)newer;
#endif
}

// Where the chunk stream of a run of FP16/FP8 products stands.
struct LoCursor {
    Product pr;     // product being staged
    int L, c, n;    // its reduction tile, the next chunk to stage, chunks per product
};

// Prepare an operand for this path: this lane's address in chunk 0, DMA instruction 0.
__device__ __forceinline__ void lo_operand(Operand &o, int q, int row0, int nb, const LoGeom &LG)
{
    if (o.p == q) {
        o.voff = (((row0 + LG.dma_row) * nb) << (3 - q)) + LG.dma_seg;
        o.sub = 0;
    }
}
__device__ __forceinline__ void lo_operand(Operand &o, int q, int row0, int nb, const LoGeom &LG, const MixGeom &MG)
{
    if (o.p == q) o.voff = (((row0 + LG.dma_row) * nb) << (3 - q)) + LG.dma_seg;
    else o.voff = (row0 + MG.row) * nb + MG.seg;                // FP8 operand of an FP16 product
    o.sub = 0;
}

// One buffer-load-to-LDS instruction of a chunk request: k = 0..3 are the four 8-row blocks of
// this wave's 32 rows of the A chunk, k = 4..7 those of the B chunk.  Lane l of instruction j
// writes LDS bytes [dst + 1024 j + 16 l, +16), i.e. row 8 j + l/8, slot l%8, and fetches the
// segment that belongs there.  The loads are asm because the compiler, not knowing which stage
// a later LDS read touches, would wait for all of them before every read; completion is awaited
// explicitly (lo_wait_dma) before the barrier that publishes the stage.  They write no
// register, so nothing the compiler allocates depends on their completion.
// An FP8 operand of an FP16 product (o.p != pr.q): a chunk is 64 bytes of each row, an
// instruction covers 16 rows, which are as many bytes of the tile as 8 rows of an FP16 operand
// (rows8_bytes holds for both), and instructions j = 2, 3 get a descriptor of length zero.
template <bool MIXED>
__device__ __forceinline__ void lo_dma_one(const Product &pr, int soff0, int rows8_bytes, unsigned dst, int k)
{
    const Operand &o = k < 4 ? pr.a : pr.b;
    const int j = k & 3;
    const bool narrow = MIXED && o.p != pr.q;
    const uint64_t b = (uint64_t)o.base;
    const i32x4 rsrc = {(int)(uint32_t)b, (int)((uint32_t)(b >> 32) & 0xffffu), (narrow && j >= 2) ? 0 : o.bytes, 0x00020000};
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(dst + (k < 4 ? 0u : (unsigned)kLoOperand) + 1024u * j), "v"(o.voff), "s"(rsrc),
                   "s"(__builtin_amdgcn_readfirstlane((narrow ? soff0 >> 1 : soff0) + j * rows8_bytes))
                 : "memory", "m0");
#else
    (void)rsrc; (void)soff0; (void)rows8_bytes; (void)dst; (void)j;
#endif
}

// Fragment registers of one chunk: index (operand * 4 + row block) * 2 + half; operand 0 = A.
// Two sets: while the MFMAs of a chunk run from one, the fragments of the next chunk (already
// published in its ring stage) are read into the other.  Read r = 0..15 of a chunk: B first.
__device__ __forceinline__ void lo_read_one(u32x4 (&f)[16], const char *stage, const LoGeom &LG, int r)
{
    constexpr int kBlock = 16 * kRowBytes;
    const int op = r < 8 ? 1 : 0, t = (r & 7) >> 1, half = r & 1;
    const int o = op ? (half ? LG.fb1 : LG.fb0) : (half ? LG.fa1 : LG.fa0);
    f[(op * 4 + t) * 2 + half] = *(const u32x4 *)(stage + o + t * kBlock);
}
__device__ __forceinline__ void lo_read_slot(u32x4 (&f)[16], const char *stage, const LoGeom &LG, int slot)
{
#pragma unroll
    for (int r = 4 * slot; r < 4 * slot + 4; ++r) lo_read_one(f, stage, LG, r);
}

// FP16 product with an FP8 operand (MIX = 1: A, 2: B).  Row block t of that operand: the lane's
// 16 bytes hold its fragment of k-step 0 (bytes 0..7) and of k-step 1 (bytes 8..15).
template <int MIX>
__device__ __forceinline__ u32x4 lo_read_narrow(const char *stage, const MixGeom &MG, int t)
{
    return *(const u32x4 *)(stage + (MIX == 1 ? MG.ma : MG.mb) + (t >> 1) * 4096 + (t & 1) * 1024);
}
// Conversion i = 0..31 of a chunk: two FP8 bytes of row block i / 8 become one register of FP16 pairs.
// BFQ: a BF16 product, the FP8 bytes become BF16 pairs (as exact: every e4m3 number is a BF16 number).
template <int MIX, bool BFQ>
__device__ __forceinline__ void lo_convert_one(u32x4 (&f)[16], const u32x4 (&raw)[4], int i)
{
    const int t = i >> 3, kk = (i >> 2) & 1, word = (i >> 1) & 1, sel = i & 1;
    const int w = (int)raw[t][2 * kk + word];
    uint32_t r;
    if constexpr (BFQ) {
        const bf2v h = sel ? __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, true) : __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, false);
        r = __builtin_bit_cast(uint32_t, h);
    } else {
        const h2v h = sel ? __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w, 1.0f, true) : __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w, 1.0f, false);
        r = __builtin_bit_cast(uint32_t, h);
    }
    f[((MIX == 1 ? 0 : 4) + t) * 2 + kk][2 * word + sel] = r;
}
// All fragments of the chunk in `stage`, outside the chunk stream (first chunk of a run, and
// where the product that follows keeps its operands differently from the one that ends).
__device__ __forceinline__ void lo_read_all(u32x4 (&f)[16], const char *stage, const LoGeom &LG, const MixGeom &MG, int mix, bool bf)
{
    if (mix == 0) {
#pragma unroll
        for (int slot = 0; slot < 4; ++slot) lo_read_slot(f, stage, LG, slot);
    } else if (mix == 1) {
        u32x4 raw[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) raw[t] = lo_read_narrow<1>(stage, MG, t);
#pragma unroll
        for (int r = 0; r < 8; ++r) lo_read_one(f, stage, LG, r);
        if (bf) {
#pragma unroll
            for (int i = 0; i < 32; ++i) lo_convert_one<1, true>(f, raw, i);
        } else {
#pragma unroll
            for (int i = 0; i < 32; ++i) lo_convert_one<1, false>(f, raw, i);
        }
    } else {
        u32x4 raw[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) raw[t] = lo_read_narrow<2>(stage, MG, t);
#pragma unroll
        for (int r = 8; r < 16; ++r) lo_read_one(f, stage, LG, r);
        if (bf) {
#pragma unroll
            for (int i = 0; i < 32; ++i) lo_convert_one<2, true>(f, raw, i);
        } else {
#pragma unroll
            for (int i = 0; i < 32; ++i) lo_convert_one<2, false>(f, raw, i);
        }
    }
}

// One step of the chunk stream: the MFMAs of a chunk from fragment set PAR.  These MFMAs leave
// issue slots free while they execute (16 or 32 cycles each), and everything else the step has
// to do is placed into those slots, one or two instructions behind each MFMA: first the reads
// of the next chunk's fragments from the ring stage `next` into the other set, then the eight
// DMA instructions that request a later chunk of product `pr` into the stage at `dst`, and the
// scalar bookkeeping of the step (`book`, straight-line code).
// The MFMAs are asm in place, see mfma_group.
// MIX != 0 (FP16 product with an FP8 operand): the next chunk's reads are the four of the FP8
// operand, then the eight of the other one; the 32 conversions follow two per MFMA.
// BFQ: the product multiplies BF16 numbers (operands as for FP16, the other matrix instruction).
template <int Q, int PAR, bool FIRST, bool MIXED, int MIX, bool BFQ, typename Book>
__device__ __forceinline__ void lo_chunk(f4 (&acc)[4][4], u32x4 (&fr)[2][16], const char *next, const LoGeom &LG, const MixGeom &MG,
                                         const Product &pr, int soff0, int rows8_bytes, unsigned dst, Book book)
{
    constexpr int kMfmas = Q == Q16 ? 32 : 16;
    u32x4 raw[4];
    constexpr int kBookSlot = Q == Q16 ? 26 : 13;    // a slot with little else in it
#pragma unroll
    for (int m = 0; m < kMfmas; ++m) {
        const int g = m >> 2, nt = m & 3, mt = g & 3, kk = g >> 2;
        const bool first = m == 0, last = m == kMfmas - 1;
        // FIRST: the product's first chunk starts its accumulators from zero (C operand 0)
        const bool zero = FIRST && (Q == Q8 || m < 16);
        if constexpr (Q == Q16 && BFQ) {
            const u32x4 x = fr[PAR][mt * 2 + kk], y = fr[PAR][(4 + nt) * 2 + kk];
            if (zero) {
                if (first) asm volatile("s_nop 3\n\tv_mfma_f32_16x16x32_bf16 %0, %1, %2, 0" : "=a"(acc[mt][nt]) : "v"(x), "v"(y));
                else asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, 0" : "=a"(acc[mt][nt]) : "v"(x), "v"(y));
            } else {
                if (first) asm volatile("s_nop 3\n\tv_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[mt][nt]) : "v"(x), "v"(y));
                else if (last) asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0\n\ts_nop 11" : "+a"(acc[mt][nt]) : "v"(x), "v"(y));
                else asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[mt][nt]) : "v"(x), "v"(y));
            }
        } else if constexpr (Q == Q16) {
            const u32x4 x = fr[PAR][mt * 2 + kk], y = fr[PAR][(4 + nt) * 2 + kk];
            if (zero) {
                if (first) asm volatile("s_nop 3\n\tv_mfma_f32_16x16x32_f16 %0, %1, %2, 0" : "=a"(acc[mt][nt]) : "v"(x), "v"(y));
                else asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, 0" : "=a"(acc[mt][nt]) : "v"(x), "v"(y));
            } else {
                if (first) asm volatile("s_nop 3\n\tv_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(acc[mt][nt]) : "v"(x), "v"(y));
                else if (last) asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0\n\ts_nop 11" : "+a"(acc[mt][nt]) : "v"(x), "v"(y));
                else asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(acc[mt][nt]) : "v"(x), "v"(y));
            }
        } else {
            const u32x4 a0 = fr[PAR][mt * 2], a1 = fr[PAR][mt * 2 + 1], b0 = fr[PAR][(4 + nt) * 2], b1 = fr[PAR][(4 + nt) * 2 + 1];
            const i8v x = {(int)a0.x, (int)a0.y, (int)a0.z, (int)a0.w, (int)a1.x, (int)a1.y, (int)a1.z, (int)a1.w};
            const i8v y = {(int)b0.x, (int)b0.y, (int)b0.z, (int)b0.w, (int)b1.x, (int)b1.y, (int)b1.z, (int)b1.w};
            // 16x16x128, both operands e4m3 (format selectors 0), no block scaling
            if (zero) {
                if (first) asm volatile("s_nop 3\n\tv_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, 0" : "=a"(acc[mt][nt]) : "v"(x), "v"(y));
                else if (last) asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, 0\n\ts_nop 11" : "=a"(acc[mt][nt]) : "v"(x), "v"(y));
                else asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, 0" : "=a"(acc[mt][nt]) : "v"(x), "v"(y));
            } else {
                if (first) asm volatile("s_nop 3\n\tv_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0" : "+a"(acc[mt][nt]) : "v"(x), "v"(y));
                else if (last) asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0\n\ts_nop 11" : "+a"(acc[mt][nt]) : "v"(x), "v"(y));
                else asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0" : "+a"(acc[mt][nt]) : "v"(x), "v"(y));
            }
        }
        SCHED_FENCE();
        if (m == kBookSlot) book();                  // the step's scalar bookkeeping (branch-free)
        if constexpr (Q == Q16 && MIX != 0) {
            if (m < 4) raw[m] = lo_read_narrow<MIX>(next, MG, m);
            else if (m < 12) lo_read_one(fr[PAR ^ 1], next, LG, (MIX == 1 ? 0 : 8) + m - 4);
            if (m >= 8 && m < 24) {
                lo_convert_one<MIX, BFQ>(fr[PAR ^ 1], raw, 2 * (m - 8));
                lo_convert_one<MIX, BFQ>(fr[PAR ^ 1], raw, 2 * (m - 8) + 1);
            }
            if (m >= 16 && m < 24) lo_dma_one<MIXED>(pr, soff0, rows8_bytes, dst, m - 16);
        } else if constexpr (Q == Q16) {
            if (m < 16) lo_read_one(fr[PAR ^ 1], next, LG, m);
            else if (m < 24) lo_dma_one<MIXED>(pr, soff0, rows8_bytes, dst, m - 16);
        } else {
            if (m < 8) {
                lo_read_one(fr[PAR ^ 1], next, LG, 2 * m);
                lo_read_one(fr[PAR ^ 1], next, LG, 2 * m + 1);
            } else {
                lo_dma_one<MIXED>(pr, soff0, rows8_bytes, dst, m - 8);
            }
        }
        SCHED_FENCE();
    }
}

template <typename AccS, bool BLOCKWISE = false>
__device__ __forceinline__ void fold(AccS (&s)[4][4], const f4 (&t)[4][4], int esum);

// A per-product FP32 accumulator set to zero.  (The compiler keeps one zero vector for the whole
// kernel, which in the FP64-tile instances is spilled and comes back from scratch memory at every
// product.  Writing the registers with immediates instead removes two thirds of that kernel's
// spills and is 0.4 % slower on cov16k and random8k, so the assignment stays.)
__device__ __forceinline__ void zero_side(f4 (&t)[4][4])
{
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) t[i][j] = f4{0, 0, 0, 0};
}

// A run of consecutive ring products starting at product `cur` (reduction tile L).  On return
// `cur` is the first product after the run (q = -1: none) and L its index; if that product wants
// its first chunk staged, it is in stage 0 of the two-stage layout.
template <typename AccS, bool MIXED, bool BF>
__device__ __forceinline__ void lo_run(AccS (&s)[4][4], Product &cur, int &L, const Walk &W, char *lds, const Geometry &G0,
                                       const Region &R)
{
    const Geometry G = fresh(G0);
    const LoGeom LG = lo_geometry(G);
    MixGeom MG{};
    if constexpr (MIXED) MG = mix_geometry(G);
    auto prepare = [&](Operand &o, int q, int row0) __attribute__((always_inline)) {
        if constexpr (MIXED) lo_operand(o, q, row0, R.nb, LG, MG);
        else lo_operand(o, q, row0, R.nb, LG);
    };
    const int wave = G.tid >> 6;
    f4 t[4][4];               // set by the first chunk of every product

    // staging cursor
    LoCursor pf;
    pf.pr = cur;
    pf.L = L;
    pf.c = 0;
    pf.n = R.nb / chunk_elems(cur.q);
    prepare(pf.pr.a, pf.pr.q, R.arow0);
    prepare(pf.pr.b, pf.pr.q, R.brow0);
    bool pf_valid = true;
    // Descriptors of the product after the one being staged: opened one product ahead so that the
    // latency of the table reads is not paid when the cursor moves on.  When the run ends this is
    // the first product that does not belong to it.
    Product nx = open_product(W.I, W.J, W.tileC, L + 1, G, R);
    bool need_open = false;
    int staged = 0;           // chunks requested so far
    int st_req = 0;           // ring stage (byte offset) of the next request
    const int wave_off = uni(wave * 4096);

    // A request = eight DMA instructions per wave (chunk pf.c of product pf.pr into the stage at
    // st_req).  Every step of the stream issues one, so that the number of outstanding
    // instructions is the same at every step; past the end of the stream the requests are
    // empty: the operands' descriptors get length zero, which turns every lane's load into an
    // out-of-range one that touches no global memory (it zero-fills its 16 bytes of a stage
    // nobody reads any more).
    // The bookkeeping after a request is split in two: `advance` is straight-line scalar code
    // (it runs in the shadow of the step's MFMAs) and only decides whether `turn` is needed,
    // the rare part with loads and branches that opens the product after next or moves the
    // cursor to the next product.
    int done = 0;                                  // chunks computed
    int st_next = kLoStage;                        // ring stage of chunk done + 1
    bool slow = false;
    auto advance = [&]() __attribute__((always_inline)) {
        st_req = st_req + kLoStage == kLoLdsBytes ? 0 : st_req + kLoStage;
        staged += pf_valid ? 1 : 0;
        pf.c += 1;
        slow = need_open || (pf_valid && pf.c == pf.n);
    };
    auto turn = [&]() __attribute__((always_inline)) {
        if (need_open) {                            // second step of a product: look one product ahead
            nx = open_product(W.I, W.J, W.tileC, pf.L + 1, G, R);
            need_open = false;
        }
        if (pf_valid && pf.c == pf.n) {             // next product: does it continue the run?
            ++pf.L;
            if (is_ring<MIXED>(nx, G)) {
                pf.pr = nx;
                prepare(pf.pr.a, nx.q, R.arow0);
                prepare(pf.pr.b, nx.q, R.brow0);
                pf.n = R.nb / chunk_elems(nx.q);
                need_open = true;
            } else {
                pf_valid = false;
                pf.pr.a.bytes = 0;
                pf.pr.b.bytes = 0;
            }
            pf.c = 0;
        }
    };
#define GMP_LO_REQ_ARGS pf.pr, pf.c * kRowBytes, (8 * R.nb) << (3 - pf.pr.q), (unsigned)(st_req + wave_off)

    // prologue: chunks 0..4 requested; chunks 0 and 1 complete and published; fragments of chunk 0 read
#pragma unroll 1
    for (int i = 0; i < kLoStages; ++i) {
#pragma unroll
        for (int k = 0; k < 8; ++k) lo_dma_one<MIXED>(GMP_LO_REQ_ARGS, k);
        advance();
        if (slow) turn();
    }
    lo_wait_dma(8 * (kLoStages - 2));
    __syncthreads();
    u32x4 fr[2][16];
    int cmix = MIXED ? ring_mix(cur.q, cur.a.p, cur.b.p) : 0;
    bool cbf = false;              // the product being computed is a BF16 one (flag in its table record)
    if constexpr (BF) cbf = ((((ConstQuad)(uintptr_t)(R.prod + L))[1].z >> 26) & 1u) != 0;
    if constexpr (MIXED) lo_read_all(fr[0], lds, LG, MG, cmix, BF && cbf);
    else {
#pragma unroll
        for (int slot = 0; slot < 4; ++slot) lo_read_slot(fr[0], lds, LG, slot);
    }

    // compute: product by product; inside a product the accumulators are touched by MFMAs only
    int cL = L;
    int cq = cur.q;
    int cesum = cur.a.e + cur.b.e;
    // One step: the MFMAs of chunk `done` from fragment set PAR; in their shadow the fragments of
    // chunk done + 1 are read from the ring stage after it (past the end of the stream that read
    // is harmless and unused) and chunk done + 5 is requested into the stage that chunk `done`
    // occupied (every wave finished reading it before the barrier that ended the previous step).
    // Then wait until chunk done + 2 is complete in LDS for every wave: everything but the three
    // requests after it.
    auto step_book = [&]() __attribute__((always_inline)) {
        advance();
        ++done;
        st_next = st_next + kLoStage == kLoLdsBytes ? 0 : st_next + kLoStage;
    };
#define GMP_LO_STEP(QQ, PAR, FIRST, MIX) GMP_LO_STEP_AS(QQ, PAR, FIRST, MIX, false)
#define GMP_LO_STEP_AS(QQ, PAR, FIRST, MIX, BFQ)                                     \
    do {                                                                             \
        lo_chunk<QQ, PAR, FIRST, MIXED, MIX, BFQ>(t, fr, lds + st_next, LG, MG, GMP_LO_REQ_ARGS, step_book); \
        if (slow) turn();                                                            \
        lo_wait_dma(8 * (kLoStages - 2));                                            \
        __syncthreads();                                                             \
    } while (0)
    while (done < staged) {
        const int cn = R.nb / chunk_elems(cq);
        // precision and exponent sum of the product after this one, fetched early
        const bool more = cL + 1 < R.kt_eff;
        const u32x4 nrec = more ? ((ConstQuad)(uintptr_t)(R.prod + cL + 1))[1] : u32x4{0, 0, 0xff0000u, 0};
        const int nq = more ? (int)((nrec.z >> 16) & 0xffu) : -1;
        const int nesum = (int)nrec.x + (int)nrec.y;
        const int nmix = MIXED ? ring_mix(nq, (int)(nrec.z & 0xffu), (int)((nrec.z >> 8) & 0xffu)) : 0;
        const bool nbf = BF && ((nrec.z >> 26) & 1u) != 0;
#define GMP_LO_PRODUCT16(MIX, BFQ)                          \
    do {                                                   \
        GMP_LO_STEP_AS(Q16, 0, true, MIX, BFQ);            \
        GMP_LO_STEP_AS(Q16, 1, false, MIX, BFQ);           \
        for (int cc = 2; cc < cn; cc += 2) {               \
            GMP_LO_STEP_AS(Q16, 0, false, MIX, BFQ);       \
            GMP_LO_STEP_AS(Q16, 1, false, MIX, BFQ);       \
        }                                                  \
    } while (0)
        if (BF && cq == Q16 && cbf) {              // a BF16 product: the BF16 matrix instruction
            if (!MIXED || cmix == 0) GMP_LO_PRODUCT16(0, true);
            else if (MIXED && cmix == 1) GMP_LO_PRODUCT16(1, true);
            else if (MIXED) GMP_LO_PRODUCT16(2, true);
        } else if (cq == Q16) {                    // 64 elements per chunk: always an even count
            if (!MIXED || cmix == 0) GMP_LO_PRODUCT16(0, false);
            else if (MIXED && cmix == 1) GMP_LO_PRODUCT16(1, false);
            else if (MIXED) GMP_LO_PRODUCT16(2, false);
        } else {
            GMP_LO_STEP(Q8, 0, true, 0);
            if (cn > 1) {
                GMP_LO_STEP(Q8, 1, false, 0);
                for (int cc = 2; cc + 2 <= cn; cc += 2) {
                    GMP_LO_STEP(Q8, 0, false, 0);
                    GMP_LO_STEP(Q8, 1, false, 0);
                }
                if (cn & 1) GMP_LO_STEP(Q8, 0, false, 0);
            }
            if (cn & 1) {                          // odd count: bring the fragments back to set 0
#pragma unroll
                for (int i = 0; i < 16; ++i) fr[0][i] = fr[1][i];
            }
        }
        // the product is complete: it joins the running sum
        fold(s, t, cesum);
        // The last step read the fragments of the next product's first chunk the way this product
        // keeps its operands; where the next one keeps them differently they are read again (that
        // chunk is complete in its stage since the barrier that ended the step).
        if constexpr (MIXED)
            if ((nmix != cmix || (BF && nmix != 0 && nbf != cbf)) && done < staged)
                lo_read_all(fr[0], lds + (st_next == 0 ? kLoLdsBytes - kLoStage : st_next - kLoStage), LG, MG, nmix, BF && nbf);
        ++cL;
        cq = nq;
        cmix = nmix;
        cbf = nbf;
        cesum = nesum;
    }
#undef GMP_LO_PRODUCT16
#undef GMP_LO_STEP
#undef GMP_LO_STEP_AS
#undef GMP_LO_REQ_ARGS
    lo_wait_dma(0);                                // the empty requests still write (zeros) into the ring
    __syncthreads();

    L = cL;
    cur = nx;
    if (wants_first_chunk<MIXED>(nx, G)) {         // hand over to the two-stage layout
        Raw xa[4], xb[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) load_pair(xa[j], xb[j], nx, R.nb, 0, j);
#pragma unroll
        for (int j = 0; j < 4; ++j) store_pair_any(xa[j], xb[j], nx, G, lds, j);
        __syncthreads();
    }
}

// ---- FP16 / FP8 products outside the ring: two-stage loop, conversion in registers ----------
// Used for FP16 products with an FP8 operand (exact FP8 -> FP16 conversion).  One chunk = 2 k-steps
// of 16x16x32 FP16, or one 16x16x128 FP8 step; the loads of the following chunk are in flight
// while the MFMAs of a chunk run.
template <int Q>
__device__ __forceinline__ void mma_padded(f4 (&acc)[4][4], const char *lds, int stage, const Geometry &G)
{
    const FragBase F = frag_base<Q>(lds + stage * kStage, G);
    constexpr int kBlock = 16 * kRowStride;
    u32x2 a[4][4], b[4][4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            a[t][w] = lds_load8(F.a + t * kBlock + 8 * w);
            b[t][w] = lds_load8(F.b + t * kBlock + 8 * w);
        }
    if constexpr (Q == Q16) {
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                for (int nt = 0; nt < 4; ++nt) {
                    const h8 x = __builtin_bit_cast(h8, u32x4{a[mt][2 * kk].x, a[mt][2 * kk].y, a[mt][2 * kk + 1].x, a[mt][2 * kk + 1].y});
                    const h8 y = __builtin_bit_cast(h8, u32x4{b[nt][2 * kk].x, b[nt][2 * kk].y, b[nt][2 * kk + 1].x, b[nt][2 * kk + 1].y});
                    if (kk == 0 && mt == 0 && nt == 0)
                        asm volatile("s_nop 3\n\tv_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(acc[mt][nt]) : "v"(x), "v"(y));
                    else if (kk == 1 && mt == 3 && nt == 3)
                        asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0\n\ts_nop 11" : "+a"(acc[mt][nt]) : "v"(x), "v"(y));
                    else
                        asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(acc[mt][nt]) : "v"(x), "v"(y));
                }
    } else {
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) {
                const i8v x = {(int)a[mt][0].x, (int)a[mt][0].y, (int)a[mt][1].x, (int)a[mt][1].y,
                               (int)a[mt][2].x, (int)a[mt][2].y, (int)a[mt][3].x, (int)a[mt][3].y};
                const i8v y = {(int)b[nt][0].x, (int)b[nt][0].y, (int)b[nt][1].x, (int)b[nt][1].y,
                               (int)b[nt][2].x, (int)b[nt][2].y, (int)b[nt][3].x, (int)b[nt][3].y};
                // 16x16x128, both operands e4m3 (format selectors 0), no block scaling
                if (mt == 0 && nt == 0)
                    asm volatile("s_nop 3\n\tv_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0" : "+a"(acc[mt][nt]) : "v"(x), "v"(y));
                else if (mt == 3 && nt == 3)
                    asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0\n\ts_nop 11" : "+a"(acc[mt][nt]) : "v"(x), "v"(y));
                else
                    asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0" : "+a"(acc[mt][nt]) : "v"(x), "v"(y));
            }
    }
}

template <int Q, int PA, int PB>
__device__ __forceinline__ void simple_chunks(f4 (&acc)[4][4], const Product &cur, int n, char *lds, int &stage, const Geometry &G, int nb)
{
    Raw ra[4], rb[4];
    Product cp = cur;
    cp.a.p = PA;
    cp.b.p = PB;
    for (int c = 1; c < n; ++c) {
#pragma unroll
        for (int j = 0; j < 4; ++j) load_pair(ra[j], rb[j], cp, nb, c, j);
        mma_padded<Q>(acc, lds, stage, G);
#pragma unroll
        for (int j = 0; j < 4; ++j) store_pair<Q>(ra[j], rb[j], cp, G, lds + (stage ^ 1) * kStage, j);
        __syncthreads();
        stage ^= 1;
    }
}

// On entry LDS stage `stage` holds the product's first chunk; on exit it holds the first chunk
// of the next product if that one wants it.
template <int Q, bool MIXED>
__device__ __forceinline__ Product product_loop_simple(f4 (&acc)[4][4], const Product &cur, const Walk &W, int Lnext, char *lds, int &stage,
                                                       const Geometry &G0, const Region &R)
{
    const Geometry G = fresh(G0);
    const int n = R.nb / chunk_elems(Q);
    if constexpr (Q == Q8) {
        simple_chunks<Q8, Q8, Q8>(acc, cur, n, lds, stage, G, R.nb);
    } else {
        if (cur.a.p == Q16 && cur.b.p == Q16) simple_chunks<Q16, Q16, Q16>(acc, cur, n, lds, stage, G, R.nb);
        else if (cur.a.p == Q16) simple_chunks<Q16, Q16, Q8>(acc, cur, n, lds, stage, G, R.nb);
        else if (cur.b.p == Q16) simple_chunks<Q16, Q8, Q16>(acc, cur, n, lds, stage, G, R.nb);
        else simple_chunks<Q16, Q8, Q8>(acc, cur, n, lds, stage, G, R.nb);
    }
    Raw ra[4], rb[4];
    const Product next = open_product(W.I, W.J, W.tileC, Lnext, G, R);
    const bool give = wants_first_chunk<MIXED>(next, G);
    if (give) {
#pragma unroll
        for (int j = 0; j < 4; ++j) load_pair(ra[j], rb[j], next, R.nb, 0, j);
    }
    mma_padded<Q>(acc, lds, stage, G);
    acc_fence<-1>(acc);
    if (give) {
#pragma unroll
        for (int j = 0; j < 4; ++j) store_pair_any(ra[j], rb[j], next, G, lds + (stage ^ 1) * kStage, j);
    }
    __syncthreads();
    stage ^= 1;
    return next;
}

// The finished tile product joins the running sum once: s += 2^esum * t.
// BLOCKWISE (FP64 sums kept in accumulation registers, which the vector ALU cannot address): each
// block of four sums completes the round trip read - add - write back before the next one sets
// out; left to itself the compiler reads all 128 registers first and spills what else is live.
template <typename AccS, bool BLOCKWISE>
__device__ __forceinline__ void fold(AccS (&s)[4][4], const f4 (&t)[4][4], int esum)
{
    constexpr bool kDouble = std::is_same<AccS, d4>::value;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if constexpr (BLOCKWISE && kDouble) {
                d4 x = s[i][j];
                asm volatile("" : "+v"(x));
#pragma unroll
                for (int v = 0; v < 4; ++v) x[v] = x[v] + ldexp((double)t[i][j][v], esum);
                asm volatile("" : "+v"(x));
                s[i][j] = x;
                asm volatile("" : "+a"(s[i][j]));
                continue;
            }
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                if constexpr (kDouble) s[i][j][v] = s[i][j][v] + ldexp((double)t[i][j][v], esum);
                else s[i][j][v] = s[i][j][v] + ldexpf(t[i][j][v], esum);
            }
        }
}

// T = double: FP64 C tiles; the running sum s is FP64 and every product below FP64 is formed
//             in the FP32 accumulator t first.
// T = float : FP32 C tiles; FP32 products continue s, FP16 / FP8 products go through t.
// LOW (T = double only): the instance for FP64 C tiles none of whose products is FP64 (a
//             covariance matrix whose tiles the norm rule stores in FP32 / FP16 throughout).  It
//             carries no FP64 product loop, which leaves the registers for what the FP32-tile kernel
//             does: the per-product accumulator in the pinned vector registers, and the next
//             product's first chunk handed over in registers and converted by that product's own
//             specialised loop.
template <typename T, bool MIXED, bool BF, bool LOW>
__device__ __forceinline__ void owner_body(const WorkItem *__restrict__ items)
{
    static_assert(!LOW || std::is_same<T, double>::value, "LOW is an instance for FP64 C tiles");
    using AccS = typename std::conditional<std::is_same<T, double>::value, d4, f4>::type;
    constexpr int QT = std::is_same<T, double>::value ? Q64 : Q32;
    extern __shared__ __attribute__((aligned(16))) char lds[];

    const Geometry G = make_geometry((int)threadIdx.x, true);

    // this workgroup's item and the kernel arguments it needs throughout: scalar loads
    const uint64_t itw = table_u64((const uint64_t *)items, blockIdx.x);
    const int tileC = (int)(uint32_t)itw;
    const ArgsPtr K0 = args();
    const int NT = K0->NT;
    const int I = tileC / NT, J = tileC % NT;
    Region R;
    R.nb = K0->nb;
    R.kt_eff = K0->kt_eff;
    R.arow0 = (int)((itw >> 32) & 0xffffu) * kMacro;
    R.brow0 = (int)((itw >> 48) & 0xffffu) * kMacro;
    R.prod = K0->prod + (int64_t)tileC * K0->KT;

    AccS s[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) s[i][j] = AccS{0, 0, 0, 0};

    int stage = 0;
    Product cur = open_product(I, J, tileC, 0, G, R);
    if (wants_first_chunk<MIXED>(cur, G)) {
        Raw ra[4], rb[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) load_pair(ra[j], rb[j], cur, R.nb, 0, j);
#pragma unroll
        for (int j = 0; j < 4; ++j) store_pair_any(ra[j], rb[j], cur, G, lds, j);
    }
    __syncthreads();

    Raw hand[8];                                   // chunk 0 of an FP64 / FP32 product on its way from
    bool raw = false;                              // its predecessor's last chunk to its own loop
    Walk W;
    W.I = I;
    W.J = J;
    W.tileC = tileC;
    int L = 0;
    while (L < R.kt_eff) {
        const int q = cur.q;
        if (is_ring<MIXED>(cur, G)) {
            lo_run<AccS, MIXED, BF>(s, cur, L, W, lds, G, R);   // all consecutive products of that kind
            stage = 0;
            continue;
        }
        Product next;
        // (No schedule the host makes comes here any more: every FP16 / FP8 product is a ring product
        // of the instance launched.  The loop stays as the road for a product no ring takes; taking
        // it out also changed the register allocation of another instance into one that the
        // build's check of the machine code rejects.)
        if (q == Q16 || q == Q8) {                 // FP16 / FP8 product outside the ring
            f4 t[4][4];
            zero_side(t);
            const int esum = cur.a.e + cur.b.e;
            if (q == Q16) next = product_loop_simple<Q16, MIXED>(t, cur, W, L + 1, lds, stage, G, R);
            else next = product_loop_simple<Q8, MIXED>(t, cur, W, L + 1, lds, stage, G, R);
            fold(s, t, esum);
            cur = next;
            ++L;
            continue;
        }
        // (only the instance for the formats beyond FP64 / FP32 / FP16 / FP8 carries the widening loop:
        // the host launches it whenever some product outside the 256 x 256 regions has such an operand)
        const bool widening = BF && is_widening(cur);
        if (LOW && q == QT) {
            next = cur;                            // not reachable: the host launches this instance only without FP64 products
            next.q = -1;
        } else if (q == QT) {
            if (BF && widening) next = product_loop_widening<QT, (QT == Q32 ? 192 : -1), MIXED>(s, cur, W, L + 1, lds, stage, G, R, raw);
            else next = product_loop_pipelined<QT, (QT == Q32 ? 192 : -1), (QT == Q32 ? 1 : 0), MIXED>(s, cur, W, L + 1, lds, stage, G, R, hand, raw);
        } else {
            if constexpr (QT == Q64 && LOW) {
                f4 t[4][4];
                zero_side(t);
                next = product_loop_pipelined<Q32, 192, 2, MIXED>(t, cur, W, L + 1, lds, stage, G, R, hand, raw);
                fold<AccS, true>(s, t, 0);
            } else if constexpr (QT == Q64) {
                // an FP32 product of an FP64 C tile: its FP32 accumulator lives only for that product
                f4 t[4][4];
                zero_side(t);
                if (BF && widening) next = product_loop_widening<Q32, -1, MIXED>(t, cur, W, L + 1, lds, stage, G, R, raw);
                else next = product_loop_pipelined<Q32, -1, 0, MIXED>(t, cur, W, L + 1, lds, stage, G, R, hand, raw);
                fold(s, t, 0);
            } else {
                next = cur;                        // not reachable: the host never schedules FP64 products on FP32 tiles
                next.q = -1;
            }
        }
        cur = next;
        ++L;
    }

    // Epilogue: v = alpha*s (+ beta*c0): two rounded products and one rounded sum in T.  C is
    // written with streaming stores: a region is written once and not read again, and should not
    // displace the operand panels from L2.
#ifdef GMP_PLAIN_C_STORES
#define GMP_STORE_C(v, p) (*(p) = (v))
#else
#define GMP_STORE_C(v, p) __builtin_nontemporal_store((v), (p))
#endif
    const ArgsPtr K = args();
    const T alpha = (T)K->alpha, beta = (T)K->beta;
    const bool use_c = K->beta != 0.0;
    if constexpr (std::is_same<T, double>::value) {
        // FP64 tiles: straight from the accumulators (8-byte stores, 128 contiguous bytes per 16
        // lanes).  The staged form below costs this kernel registers it does not have: measured
        // 1 % slower overall, while its C traffic is negligible against 64-cycle MFMAs.
        typedef __attribute__((address_space(1))) T *GlobalT;
        GlobalT ctile = (GlobalT)(uintptr_t)(K->C.storage + table_u64(K->C.offset, tileC));
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int row = R.arow0 + G.wm * 64 + mt * 16 + 4 * G.g + v;
                    const int col = R.brow0 + G.wn * 64 + nt * 16 + G.li;
                    GlobalT p = ctile + (int64_t)row * R.nb + col;
                    T val = alpha * (T)s[mt][nt][v];
                    if (use_c) { const T bc = beta * *p; val = val + bc; }
                    GMP_STORE_C(val, p);
                }
    } else {
        // FP32 tiles: the accumulator layout (a lane holds a 4-row column piece of each 16x16
        // block) would make 4-byte stores scattered over four rows; each wave therefore turns
        // its 64 x 64 block through a private, padded piece of LDS (the operand stages are dead
        // by now) and moves 16 bytes per lane along the rows: whole 256-byte row segments per
        // instruction, for the C tile read by beta as well.
        constexpr int kVec = 16 / (int)sizeof(T);                    // elements per lane and pass: 4 or 2
        constexpr int kLanesPerRow = 64 / kVec;                      // 16 or 32
        constexpr int kRowsPerPass = 64 / kLanesPerRow;              // 4 or 2
        constexpr int kEpiStride = 64 + kVec;                        // row pitch in elements: 272 or 528 bytes
        typedef T VecT __attribute__((ext_vector_type(kVec)));
        typedef __attribute__((address_space(1))) VecT *GlobalVec;
        __syncthreads();                                             // every wave is done with the stages
        T *stg = (T *)lds + (G.tid >> 6) * (64 * kEpiStride);
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt)
#pragma unroll
                for (int v = 0; v < 4; ++v) stg[(mt * 16 + 4 * G.g + v) * kEpiStride + nt * 16 + G.li] = (T)s[mt][nt][v];
        const int er = G.lane / kLanesPerRow, ec = (G.lane % kLanesPerRow) * kVec;
        const char *cbase = K->C.storage + table_u64(K->C.offset, tileC)
                            + ((int64_t)(R.arow0 + G.wm * 64 + er) * R.nb + R.brow0 + G.wn * 64 + ec) * (int64_t)sizeof(T);
        const int64_t pass_bytes = (int64_t)kRowsPerPass * R.nb * (int64_t)sizeof(T);
#pragma unroll 4
        for (int pass = 0; pass < 64 / kRowsPerPass; ++pass) {
            const VecT sv = *(const VecT *)&stg[(pass * kRowsPerPass + er) * kEpiStride + ec];
            GlobalVec gp = (GlobalVec)(uintptr_t)(cbase + pass * pass_bytes);
            VecT val;
#pragma unroll
            for (int i = 0; i < kVec; ++i) val[i] = alpha * sv[i];
            if (use_c) {
                const VecT c0 = *gp;
#pragma unroll
                for (int i = 0; i < kVec; ++i) { const T bc = beta * c0[i]; val[i] = val[i] + bc; }
            }
            GMP_STORE_C(val, gp);
        }
    }
}

}  // namespace gmp

// One instance per translation unit: its set-up call (the dynamic LDS size must be raised once
// per kernel) and its launcher.
namespace gmp {
template <typename T, bool MIXED, bool BF>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(1, 1)))
void gemm_mp_owner_kernel(GemmArgs P, const WorkItem *__restrict__ items)
{
    (void)P;                                       // read through the kernel argument segment (args())
    owner_body<T, MIXED, BF, false>(items);
}
// FP64 C tiles without an FP64 product (see owner_body).  A template only so that the one
// translation unit that names it compiles it; MIXED: as for the other instances.
template <bool MIXED>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(1, 1)))
void gemm_mp_owner_low_kernel(GemmArgs P, const WorkItem *__restrict__ items)
{
    (void)P;
    owner_body<double, MIXED, false, true>(items);
}
}  // namespace gmp

#define GMP_OWNER_INSTANCE(NAME, T, MIXED, BF)                                                              \
    namespace gmp {                                                                                         \
    hipError_t setup_##NAME()                                                                               \
    {                                                                                                       \
        return hipFuncSetAttribute((const void *)gemm_mp_owner_kernel<T, MIXED, BF>,                        \
                                   hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);                  \
    }                                                                                                       \
    hipError_t launch_##NAME(const GemmArgs &a, const WorkItem *items, int n, hipStream_t s)                \
    {                                                                                                       \
        gemm_mp_owner_kernel<T, MIXED, BF><<<dim3((unsigned)n), dim3(kThreads), kLdsBytes, s>>>(a, items);  \
        return hipGetLastError();                                                                           \
    }                                                                                                       \
    }
#define GMP_OWNER_LOW_INSTANCE(NAME)                                                                        \
    namespace gmp {                                                                                         \
    hipError_t setup_##NAME()                                                                               \
    {                                                                                                       \
        return hipFuncSetAttribute((const void *)gemm_mp_owner_low_kernel<false>,                                 \
                                   hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);                  \
    }                                                                                                       \
    hipError_t launch_##NAME(const GemmArgs &a, const WorkItem *items, int n, hipStream_t s)                \
    {                                                                                                       \
        gemm_mp_owner_low_kernel<false><<<dim3((unsigned)n), dim3(kThreads), kLdsBytes, s>>>(a, items);     \
        return hipGetLastError();                                                                           \
    }                                                                                                       \
    }
