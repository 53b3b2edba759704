// Owner-workgroup kernel of the tile-centric mixed-precision GEMM for gfx950 (CDNA4).
//
// One workgroup (256 threads = 4 waves as 2 x 2) owns a 128 x 128 region of one C tile for the
// whole reduction: it walks the reduction tiles L = 0..KT-1 in ascending order, runs each tile
// product A(I,L)*B(L,J) on the matrix cores at that task's precision q, and writes C once.
// Nothing else ever touches that region, so there are no atomics and the result is
// reproducible.
//
// Data path of one reduction chunk (128 bytes of converted reduction index per row, i.e.
// 16 FP64 / 32 FP32 / 64 FP16 / 128 FP8 values):
//   global (stored precision) -> registers -> convert to q ("receiver-side conversion": exact
//   up-casts with the tile's 2^e applied, or the one down-cast FP64 -> FP32) -> LDS (rows of
//   128 B + 16 B pad) -> 16x16 MFMA fragments.  The loads of the next chunk are issued before
//   the MFMAs of the current one and land in the other LDS stage afterwards; the chunk stream
//   runs across tile-product boundaries so the pipeline never drains inside a C region.
//
// Fragment convention.  Packed A tiles are row-major and packed B tiles are stored transposed,
// so both operands have the reduction index contiguous.  Lane (i = lane%16, g = lane/16) reads
// bytes [32g, 32g+32) of row i of a 16-row block for both operands; which reduction index that
// is does not matter as long as A and B agree, and they do by construction.  The accumulator
// of a 16x16 FP32-result MFMA holds C[4g+v][i] in register v; the FP64 MFMA holds C[4v+g][i],
// so on the FP64 path lane i reads A row 4*(i%4) + i/4 instead of row i, which makes both
// accumulator kinds address the same C element in the same lane and register.
#include <type_traits>

#include "gemm_mp_internal.h"

namespace gmp {

typedef double d4 __attribute__((ext_vector_type(4)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef int i8v __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // native vectors: these stay in registers
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kRowBytes = 128;                       // converted bytes per row and chunk
constexpr int kRowStride = 144;                      // + 16 B pad against LDS bank conflicts
constexpr int kOperandStage = kMacro * kRowStride;   // 18432 B
constexpr int kStage = 2 * kOperandStage;            // A then B
constexpr int kLdsBytes = 2 * kStage;                // two stages: 73728 B
constexpr int kThreads = 256;

enum { Q64 = GEMM_MP_FP64, Q32 = GEMM_MP_FP32, Q16 = GEMM_MP_FP16, Q8 = GEMM_MP_FP8_E4M3 };

// Raw (still in stored precision) data of one 16-byte converted segment.  Every segment is
// fetched with the same instruction whatever the stored precision: the aligned 16 bytes that
// contain its source (plus the next 16 for the one down-cast, FP64 -> FP32, whose source is
// 32 bytes).  Loads therefore need no control flow and are all issued back to back; when the
// source is narrower than 16 bytes, neighbouring lanes fetch the same 16 bytes and each picks
// its part at conversion time (`sub` = byte offset of the source inside the 16 bytes).
struct Raw { u32x4 lo, hi; };

typedef const __attribute__((address_space(1))) u32x4 *GlobalVec;

// 16-byte load through the global (not the flat) address space.
__device__ __forceinline__ u32x4 load16(const char *p)
{
    return *(GlobalVec)(uintptr_t)p;
}

// Q: product precision (fixes how many elements a 16-byte converted segment holds);
// p: stored precision; eidx: element index of the segment's first element in the tile.
template <int Q>
__device__ __forceinline__ void load_raw(Raw &r, const char *tile, int p, int64_t eidx)
{
    const int64_t off = eidx << (3 - p);
    r.lo = load16(tile + (off & ~(int64_t)15));
    if (Q == Q32 && p == Q64) r.hi = load16(tile + off + 16);
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

// One tile product A(I,L)*B(L,J) as the loader and the MFMA loop see it; koff is the first
// reduction index (in elements) of the chunk being loaded.
struct Chunk {
    const char *a, *b;     // tile bases
    int64_t koff;
    int pA, pB, q;
    int eA, eB;
};

struct Geometry {
    int tid, lane, li, g, wm, wn;
    int seg_row, seg_part;          // staging: this thread's first row and its 16-byte part
};

__device__ __forceinline__ int chunk_elems(int q) { return kRowBytes >> (3 - q); }   // 16, 32, 64, 128

template <int Q>
__device__ __forceinline__ void issue_loads(Raw (&ra)[4], Raw (&rb)[4], const Chunk &c, const Geometry &G,
                                   int nb, int arow0, int brow0)
{
    constexpr int n_q = 16 / (8 >> Q);   // elements per 16-byte converted segment
    // The offsets below are cheap to form and would otherwise be hoisted, for every precision
    // pair, out of the whole reduction loop and kept in registers; the empty asm pins their
    // computation here.
    int seg_row = G.seg_row, seg_part = G.seg_part;
    asm volatile("" : "+v"(seg_row), "+v"(seg_part));
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int row = seg_row + 32 * j;
        load_raw<Q>(ra[j], c.a, c.pA, (int64_t)(arow0 + row) * nb + c.koff + seg_part * n_q);
        load_raw<Q>(rb[j], c.b, c.pB, (int64_t)(brow0 + row) * nb + c.koff + seg_part * n_q);
    }
}

template <int Q>
__device__ __forceinline__ void convert_store(const Raw (&ra)[4], const Raw (&rb)[4], const Chunk &c,
                                     const Geometry &G, char *stage)
{
    constexpr int n_q = 16 / (8 >> Q);
    int seg_row = G.seg_row, seg_part = G.seg_part;
    asm volatile("" : "+v"(seg_row), "+v"(seg_part));
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int row = seg_row + 32 * j;
        // source offset inside the loaded 16 bytes: (seg_part * n_q elements * size_p) mod 16;
        // rows and chunk starts are multiples of 16 bytes in every precision
        const int subA = ((seg_part * n_q) << (3 - c.pA)) & 15, subB = ((seg_part * n_q) << (3 - c.pB)) & 15;
        *(u32x4 *)(stage + row * kRowStride + seg_part * 16) = convert<Q>(ra[j], c.pA, c.eA, subA);
        *(u32x4 *)(stage + kOperandStage + row * kRowStride + seg_part * 16) = convert<Q>(rb[j], c.pB, c.eB, subB);
    }
}

// 32 bytes of one fragment row.
struct Frag { u32x4 lo, hi; };
__device__ __forceinline__ Frag read_frag(const char *operand, int row, int g)
{
    const char *p = operand + row * kRowStride + g * 32;
    Frag f;
    f.lo = *(const u32x4 *)p;
    f.hi = *(const u32x4 *)(p + 16);
    return f;
}
__device__ __forceinline__ uint32_t frag_word(const Frag &f, int w)
{
    const u32x4 v = w < 4 ? f.lo : f.hi;
    return v[w & 3];
}

__device__ __forceinline__ void mma_fp64(d4 (&acc)[4][4], const char *stage, const Geometry &G)
{
    Frag a[4], b[4];
    const int arow = 4 * (G.li & 3) + (G.li >> 2);      // see the fragment convention above
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        a[t] = read_frag(stage, G.wm * 64 + t * 16 + arow, G.g);
        b[t] = read_frag(stage + kOperandStage, G.wn * 64 + t * 16 + G.li, G.g);
    }
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        double av[4], bv[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            av[t] = as_double(frag_word(a[t], 2 * kk), frag_word(a[t], 2 * kk + 1));
            bv[t] = as_double(frag_word(b[t], 2 * kk), frag_word(b[t], 2 * kk + 1));
        }
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt)
                acc[mt][nt] = __builtin_amdgcn_mfma_f64_16x16x4f64(av[mt], bv[nt], acc[mt][nt], 0, 0, 0);
    }
}

__device__ __forceinline__ void mma_fp32(f4 (&acc)[4][4], const char *stage, const Geometry &G)
{
    Frag a[4], b[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        a[t] = read_frag(stage, G.wm * 64 + t * 16 + G.li, G.g);
        b[t] = read_frag(stage + kOperandStage, G.wn * 64 + t * 16 + G.li, G.g);
    }
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt)
                acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(frag_word(a[mt], kk)),
                                                                   __uint_as_float(frag_word(b[nt], kk)),
                                                                   acc[mt][nt], 0, 0, 0);
    }
}

__device__ __forceinline__ void mma_fp16(f4 (&acc)[4][4], const char *stage, const Geometry &G)
{
    Frag a[4], b[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        a[t] = read_frag(stage, G.wm * 64 + t * 16 + G.li, G.g);
        b[t] = read_frag(stage + kOperandStage, G.wn * 64 + t * 16 + G.li, G.g);
    }
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) {
                const h8 x = __builtin_bit_cast(h8, kk ? a[mt].hi : a[mt].lo);
                const h8 y = __builtin_bit_cast(h8, kk ? b[nt].hi : b[nt].lo);
                acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(x, y, acc[mt][nt], 0, 0, 0);
            }
    }
}

__device__ __forceinline__ void mma_fp8(f4 (&acc)[4][4], const char *stage, const Geometry &G)
{
    Frag a[4], b[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        a[t] = read_frag(stage, G.wm * 64 + t * 16 + G.li, G.g);
        b[t] = read_frag(stage + kOperandStage, G.wn * 64 + t * 16 + G.li, G.g);
    }
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
            const i8v x = {(int)a[mt].lo.x, (int)a[mt].lo.y, (int)a[mt].lo.z, (int)a[mt].lo.w,
                           (int)a[mt].hi.x, (int)a[mt].hi.y, (int)a[mt].hi.z, (int)a[mt].hi.w};
            const i8v y = {(int)b[nt].lo.x, (int)b[nt].lo.y, (int)b[nt].lo.z, (int)b[nt].lo.w,
                           (int)b[nt].hi.x, (int)b[nt].hi.y, (int)b[nt].hi.z, (int)b[nt].hi.w};
            // 16x16x128, both operands e4m3, block scales 2^0 (E8M0 code 127)
            acc[mt][nt] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(x, y, acc[mt][nt], 0, 0, 0, 127, 0, 127);
        }
}

// Everything that describes a chunk is the same for all lanes of the workgroup; passing it
// through readfirstlane keeps it in scalar registers and makes every branch on it a scalar one.
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ const char *uni(const char *p)
{
    const uint64_t v = (uint64_t)p;
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
    return (const char *)(((uint64_t)hi << 32) | lo);
}

// Load the descriptors of tile product L of this C tile (q = -1 past the end).
__device__ __forceinline__ Chunk open_product(const GemmArgs &P, int I, int J, int tileC, int L)
{
    Chunk c;
    c.koff = 0;
    c.a = c.b = nullptr;
    c.pA = c.pB = c.eA = c.eB = 0;
    c.q = -1;
    if (L >= P.kt_eff) return c;
    const int ta = I * P.KT + L, tb = L * P.NT + J;
    c.a = uni(P.A.storage + P.A.offset[ta]);
    c.b = uni(P.B.storage + P.B.offset[tb]);
    c.pA = uni(P.A.prec[ta]);
    c.pB = uni(P.B.prec[tb]);
    c.eA = uni(P.A.exp[ta]);
    c.eB = uni(P.B.exp[tb]);
    c.q = uni(P.q[(int64_t)tileC * P.KT + L]);
    return c;
}

struct Region {
    int nb, arow0, brow0;
};

// Loads / conversion of a chunk whose precision is only known at run time (the first chunk of
// the next tile product).
__device__ __forceinline__ void issue_loads_any(Raw (&ra)[4], Raw (&rb)[4], const Chunk &c, const Geometry &G, const Region &R)
{
    switch (c.q) {
    case Q64: issue_loads<Q64>(ra, rb, c, G, R.nb, R.arow0, R.brow0); break;
    case Q32: issue_loads<Q32>(ra, rb, c, G, R.nb, R.arow0, R.brow0); break;
    case Q16: issue_loads<Q16>(ra, rb, c, G, R.nb, R.arow0, R.brow0); break;
    case Q8:  issue_loads<Q8>(ra, rb, c, G, R.nb, R.arow0, R.brow0);  break;
    default: break;
    }
}
__device__ __forceinline__ void convert_store_any(const Raw (&ra)[4], const Raw (&rb)[4], const Chunk &c, const Geometry &G, char *stage)
{
    switch (c.q) {
    case Q64: convert_store<Q64>(ra, rb, c, G, stage); break;
    case Q32: convert_store<Q32>(ra, rb, c, G, stage); break;
    case Q16: convert_store<Q16>(ra, rb, c, G, stage); break;
    case Q8:  convert_store<Q8>(ra, rb, c, G, stage);  break;
    default: break;
    }
}

template <int Q, typename Acc>
__device__ __forceinline__ void mma(Acc (&acc)[4][4], const char *stage, const Geometry &G)
{
    if constexpr (Q == Q64) mma_fp64(acc, stage, G);
    else if constexpr (Q == Q32) mma_fp32(acc, stage, G);
    else if constexpr (Q == Q16) mma_fp16(acc, stage, G);
    else mma_fp8(acc, stage, G);
}

// All chunks of one tile product at precision Q.  On entry LDS stage `stage` holds the
// product's first chunk; on exit it holds the first chunk of the next product (if any).
// While the MFMAs of a chunk run, the loads of the following chunk are in flight.
template <int Q, typename Acc>
__device__ __forceinline__ void product_loop(Acc (&acc)[4][4], Chunk cur, const Chunk &next, char *lds, int &stage,
                                    const Geometry &G, const Region &R)
{
    Raw ra[4], rb[4];
    const int n = R.nb / (kRowBytes >> (3 - Q));
    for (int c = 0; c < n - 1; ++c) {
        cur.koff += kRowBytes >> (3 - Q);
        issue_loads<Q>(ra, rb, cur, G, R.nb, R.arow0, R.brow0);
        mma<Q>(acc, lds + stage * kStage, G);
        convert_store<Q>(ra, rb, cur, G, lds + (stage ^ 1) * kStage);
        __syncthreads();
        stage ^= 1;
    }
    issue_loads_any(ra, rb, next, G, R);
    mma<Q>(acc, lds + stage * kStage, G);
    convert_store_any(ra, rb, next, G, lds + (stage ^ 1) * kStage);
    __syncthreads();
    stage ^= 1;
}

// The finished tile product joins the running sum once: s += 2^esum * t, then t = 0.
template <typename AccS>
__device__ __forceinline__ void fold(AccS (&s)[4][4], f4 (&t)[4][4], int esum)
{
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                if constexpr (std::is_same<AccS, d4>::value) s[i][j][v] = s[i][j][v] + ldexp((double)t[i][j][v], esum);
                else s[i][j][v] = s[i][j][v] + ldexpf(t[i][j][v], esum);
            }
            t[i][j] = f4{0, 0, 0, 0};
        }
}

// T = double: FP64 C tiles; the running sum s is FP64 and every product below FP64 is formed
//             in the FP32 accumulator t first.
// T = float : FP32 C tiles; FP32 products continue s, FP16 / FP8 products go through t.
template <typename T>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(1, 1)))
void gemm_mp_owner_kernel(GemmArgs P, const WorkItem *__restrict__ items)
{
    using AccS = typename std::conditional<std::is_same<T, double>::value, d4, f4>::type;
    constexpr int QT = std::is_same<T, double>::value ? Q64 : Q32;
    extern __shared__ __attribute__((aligned(16))) char lds[];

    Geometry G;
    G.tid = threadIdx.x;
    G.lane = G.tid & 63;
    G.li = G.lane & 15;
    G.g = G.lane >> 4;
    const int wave = G.tid >> 6;
    G.wm = wave >> 1;
    G.wn = wave & 1;
    G.seg_row = G.tid >> 3;
    G.seg_part = G.tid & 7;

    const WorkItem it = items[blockIdx.x];
    const int tileC = uni((int)it.tile);
    const int I = tileC / P.NT, J = tileC % P.NT;
    Region R;
    R.nb = P.nb;
    R.arow0 = uni((int)it.mi) * kMacro;
    R.brow0 = uni((int)it.mj) * kMacro;

    AccS s[4][4];
    f4 t[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            s[i][j] = AccS{0, 0, 0, 0};
            t[i][j] = f4{0, 0, 0, 0};
        }

    int stage = 0;
    Chunk cur = open_product(P, I, J, tileC, 0);
    {
        Raw ra[4], rb[4];
        issue_loads_any(ra, rb, cur, G, R);
        convert_store_any(ra, rb, cur, G, lds);
    }
    __syncthreads();

    for (int L = 0; L < P.kt_eff; ++L) {
        const Chunk next = open_product(P, I, J, tileC, L + 1);
        const int q = cur.q;
        if (q == QT) {
            product_loop<QT>(s, cur, next, lds, stage, G, R);
        } else {
            if (q == Q32) product_loop<Q32>(t, cur, next, lds, stage, G, R);
            else if (q == Q16) product_loop<Q16>(t, cur, next, lds, stage, G, R);
            else product_loop<Q8>(t, cur, next, lds, stage, G, R);
            fold(s, t, q == Q32 ? 0 : cur.eA + cur.eB);
        }
        cur = next;
    }

    // Epilogue: v = alpha*s (+ beta*c0): two rounded products and one rounded sum in T.
    T *ctile = (T *)(P.C.storage + P.C.offset[tileC]);
    const T alpha = (T)P.alpha, beta = (T)P.beta;
    const bool use_c = P.beta != 0.0;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = R.arow0 + G.wm * 64 + mt * 16 + 4 * G.g + v;
                const int col = R.brow0 + G.wn * 64 + nt * 16 + G.li;
                T *p = ctile + (int64_t)row * P.nb + col;
                T val = alpha * (T)s[mt][nt][v];
                if (use_c) { const T bc = beta * *p; val = val + bc; }
                *p = val;
            }
}

hipError_t gemm_kernel_setup()
{
    hipError_t e = hipFuncSetAttribute((const void *)gemm_mp_owner_kernel<double>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute((const void *)gemm_mp_owner_kernel<float>,
                               hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
}

// Two launches at most: the owner regions of FP64 C tiles, then those of FP32 C tiles.
hipError_t launch_gemm(const GemmArgs &a, hipStream_t s)
{
    if (a.n_items64 > 0)
        gemm_mp_owner_kernel<double><<<dim3((unsigned)a.n_items64), dim3(kThreads), kLdsBytes, s>>>(a, a.items64);
    if (a.n_items32 > 0)
        gemm_mp_owner_kernel<float><<<dim3((unsigned)a.n_items32), dim3(kThreads), kLdsBytes, s>>>(a, a.items32);
    return hipGetLastError();
}

}  // namespace gmp
