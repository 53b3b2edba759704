// Device code of the kernels with 256 x 256 regions (templates; one instance per translation unit,
// see gemm_region_*.hip).
#pragma once
#include "gemm_owner_kernel.h"

namespace gmp {

// ---- FP32 C tiles whose tile products are all FP8 x FP8: 256 x 256 regions -------------------
// At FP8 rates a 128 x 128 region asks the L2 for 64 bytes and the LDS for 128 bytes per cycle
// and CU: both paths' full width.  A C tile whose every product takes two FP8 tiles as stored
// (no conversion) is therefore cut into 256 x 256 regions: 4 waves of 128 x 128, i.e. 4 x 4
// blocks of the 32x32x64 FP8 MFMA per wave, which halves both the bytes fetched from L2 and the
// bytes read from LDS per flop, and quarters the number of workgroups and their fixed costs.
// The 256 accumulator registers of a wave leave no room for a per-product accumulator beside
// the running sum, so the tile scales are applied inside the matrix core instead: the MFMA's
// block-scale operands (an E8M0 exponent per operand) carry 2^eA and 2^eB, every product term
// enters the one FP32 accumulator at its true magnitude, and there is no fold.  (The order of
// the FP32 additions differs from the smaller regions': one chain over the whole reduction.)
// Chunks of 128 bytes per row stream through two 64 KB LDS stages by global -> LDS DMA with
// the same swizzle as the FP64 / FP32 stages; a chunk is two halves of 16 MFMAs; while a half
// runs, the fragments of the next half are read, and in the second half the requests for the
// chunk after the next go out into the stage just vacated.  One barrier per chunk, in the
// middle: it publishes the next chunk (requested a whole chunk earlier) and frees this one's.
constexpr int kBigMacro = 256;
constexpr int kBigOperand = kBigMacro * kRowBytes;     // 32 KB
constexpr int kBigStage = 2 * kBigOperand;             // A then B
constexpr int kBigLdsBytes = 2 * kBigStage;            // 128 KB
// Block-scaled formats, tiles of up to 1024: the scale bytes of a product's 256 + 256 rows travel
// through two buffers behind the stages (at most 8 KB per operand and product).
constexpr int kBigScaleOperand = 8192;
constexpr int kBigScaleBuf = 2 * kBigScaleOperand;     // A then B
constexpr int kBigLdsScaled = kBigLdsBytes + 2 * kBigScaleBuf;   // 160 KB
typedef float f16v __attribute__((ext_vector_type(16)));

struct BigGeom {
    int voff[2][2];      // [operand][instruction parity]: this lane's byte offset in a tile for DMA instruction 0 / 1
    int ra[2][2][2];     // [stage][half][which 16 bytes]: LDS address of this lane's fragment bytes, A block 0
    int rb[2][2][2];     // same for B (includes the operand offset)
    unsigned dst;        // LDS address of this wave's first DMA row of operand A, stage 0
    int rows8;           // byte distance of 8 tile rows
    int rot, n;          // chunk c of a product (n of them) is chunk (c + rot) mod n of the tile rows; rot even
};

// Scale exponents of a product as the two E8M0 operands of the MFMA (bias 127, range +-127;
// what one operand cannot hold moves to the other; beyond both the FP32 result is 0 or inf
// in any case), replicated into all four bytes.
__device__ __forceinline__ void big_scales(int ea, int eb, int &sa, int &sb)
{
    int xa = ea < -127 ? -127 : ea > 127 ? 127 : ea;
    int rest = eb + (ea - xa);
    int xb = rest < -127 ? -127 : rest > 127 ? 127 : rest;
    rest = xa + (rest - xb);
    xa = rest < -127 ? -127 : rest > 127 ? 127 : rest;
    sa = (xa + 127) * 0x01010101;
    sb = (xb + 127) * 0x01010101;
}

// DMA instruction j = 0..15 of a wave for one chunk: j < 8 moves rows 8 j .. 8 j + 7 of the
// wave's 64 rows of A, j >= 8 the same of B, 16 bytes per lane, into the stage at `dst`.
// base / bytes: the operand tile (bytes = 0: nothing is fetched, zeros are written).
__device__ __forceinline__ void big_dma_one(uint64_t base, int bytes, int voff, int soff, unsigned dst)
{
    const i32x4 rsrc = {(int)(uint32_t)base, (int)((uint32_t)(base >> 32) & 0xffffu), bytes, 0x00020000};
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(dst), "v"(voff), "s"(rsrc), "s"(soff)
                 : "memory", "m0");
#else
    (void)rsrc; (void)voff; (void)soff; (void)dst;
#endif
}
struct BigSource {
    uint64_t a, b;       // operand tiles of the product the chunk belongs to
    int bytes;           // nb * nb, or 0 past the end of the reduction
    int c;               // chunk index in that product
};
template <int FMT>
__device__ __forceinline__ void big_request(const BigSource &S, const BigGeom &BG, int stage, int j)
{
    int cc = S.c + BG.rot;
    if (cc >= BG.n) cc -= BG.n;
    if constexpr (FMT == 5) {
        // MXFP6: the 256 rows of an operand's chunk are 24 KB in one piece (a tile is stored panel by
        // panel of 128 reduction indices, see fp6_group_offset) and go to LDS as they are: twelve
        // instructions per wave and chunk, six for each operand, 1 KB each; rows8 is the size of a panel
        if (j >= 12) return;
        const int op = j >= 6, jj = op ? j - 6 : j;
        big_dma_one(op ? S.b : S.a, S.bytes, BG.voff[op][0], uni(cc * BG.rows8 + jj * 1024),
                    BG.dst + (unsigned)(stage * kBigStage + op * kBigOperand + jj * 1024));
    } else {
        const int op = j >> 3, jj = j & 7;
        big_dma_one(op ? S.b : S.a, S.bytes, BG.voff[op][jj & 1], uni(cc * kRowBytes + jj * BG.rows8),
                    BG.dst + (unsigned)(stage * kBigStage + op * kBigOperand + jj * 1024));
    }
}
// One 16-byte half (w) of fragment t (0..3: A blocks of 32 rows, 4..7: B blocks) of half `hc` of the
// chunk in `stage`, into its place in the fragment.
// A fragment is the operand of one matrix instruction: eight registers, six for FMT 5 (kept in a
// six-register type so that the two spare ones are not allocated sixteen times over): there a
// lane's block of 32 six-bit elements is 24 consecutive bytes of its row, 8-byte aligned, read as
// three pairs of registers, two with w = 0 and the third with w = 1.
typedef int i6v __attribute__((ext_vector_type(6)));
template <int FMT> struct BigFrag { typedef i8v type; };
template <> struct BigFrag<5> { typedef i6v type; };
template <int FMT>
__device__ __forceinline__ void big_read_half(typename BigFrag<FMT>::type &f, const BigGeom &BG, const char *lds, int stage, int hc, int t, int w)
{
    if constexpr (FMT == 5) {
        const char *p = lds + (t < 4 ? BG.ra[stage][hc][0] : BG.rb[stage][hc][0]) + (t & 3) * (32 * 96);
        if (w == 0) {
            const u32x2 a = *(const u32x2 *)p, b = *(const u32x2 *)(p + 8);
            f[0] = (int)a.x; f[1] = (int)a.y; f[2] = (int)b.x; f[3] = (int)b.y;
        } else {
            const u32x2 c = *(const u32x2 *)(p + 16);
            f[4] = (int)c.x; f[5] = (int)c.y;
        }
    } else {
        const char *p = lds + (t < 4 ? BG.ra[stage][hc][w] : BG.rb[stage][hc][w]) + (t & 3) * (32 * kRowBytes);
        const u32x4 v = *(const u32x4 *)p;
        f[4 * w] = (int)v.x; f[4 * w + 1] = (int)v.y; f[4 * w + 2] = (int)v.z; f[4 * w + 3] = (int)v.w;
    }
}

// The whole fragment.
template <int FMT>
__device__ __forceinline__ typename BigFrag<FMT>::type big_read(const BigGeom &BG, const char *lds, int stage, int hc, int t)
{
    if constexpr (FMT == 5) {
        i6v f = {};
        big_read_half<FMT>(f, BG, lds, stage, hc, t, 0);
        big_read_half<FMT>(f, BG, lds, stage, hc, t, 1);
        return f;
    } else {
    const char *p0 = lds + (t < 4 ? BG.ra[stage][hc][0] : BG.rb[stage][hc][0]) + (t & 3) * (32 * kRowBytes);
    const char *p1 = lds + (t < 4 ? BG.ra[stage][hc][1] : BG.rb[stage][hc][1]) + (t & 3) * (32 * kRowBytes);
    const u32x4 lo = *(const u32x4 *)p0, hi = *(const u32x4 *)p1;
    return i8v{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
    }
}
// The fragment as the eight-register value the instruction's builtin asks for (FMT 5: the two
// registers beyond the six are not read by the instruction and are left undefined).
__device__ __forceinline__ i8v big_operand(const i8v &f) { return f; }
__device__ __forceinline__ i8v big_operand(const i6v &f) { return __builtin_shufflevector(f, f, 0, 1, 2, 3, 4, 5, -1, -1); }

// Block scales of an MXFP8 chunk: per A row block (0..3) and B row block (4..7) the four scale
// bytes of this lane's row (one per 32 reduction indices of the chunk), shifted so that byte 0
// is the block this lane answers for in the chunk's first half and byte 2 in its second (the
// instruction takes the scale of the first 32 indices of its 64 from lanes 0..31 and that of
// the second 32 from lanes 32..63).
struct BigScaleGeom {
    int soa, sob;        // byte offset of this lane's scale row, A block 0 / B block 0, from the tile's start
    int shift;           // 8 * (lane / 32)
    int rot, n;          // as in BigGeom
    // scales through LDS (tiles of up to 1024: a row has at most 32 scale bytes):
    int rb;              // scale bytes per tile row, nb / 32
    int ua, ub;          // byte offset, from the tile's start, of the scale rows of the region's 256 rows of A / B
    int la, lb;          // this lane's scale row in a scale buffer, A block 0 / B block 0
    int lane16;          // 16 * lane
};
struct BigScaleTake {    // where the scale words of the following chunk pair are read from, if from LDS
    int buf, c;
};
// One call fetches the scales of the chunk pair c, c + 1 (c even) with one load per row block.
// (A wave's scale loads touch 32 different cache lines each, as costly for the vector memory path
// as two of the chunk's DMA instructions: hence as few and as wide as possible.)
// FMT 1 (MXFP8): four scale bytes per row and chunk: d[0..7] chunk c, d[8..15] chunk c + 1.
// FMT 2 (MXFP4): a chunk holds 256 reduction indices, eight scale bytes per row: d[0..7] first half
// of chunk c, d[8..15] its second half, d[16..31] the same of chunk c + 1.
template <int FMT>
__device__ __forceinline__ void big_load_scales(int (&d)[32], const BigScaleGeom &SG, uint64_t a, uint64_t b, int nb, int c)
{
    c += SG.rot;
    if (c >= SG.n) c -= SG.n;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        if constexpr (FMT == 2) {
            const u32x4 x = *(const u32x4 *)(uintptr_t)(a + (uint64_t)(SG.soa + t * nb + 8 * c));
            const u32x4 y = *(const u32x4 *)(uintptr_t)(b + (uint64_t)(SG.sob + t * nb + 8 * c));
            d[t] = (int)x.x; d[8 + t] = (int)x.y; d[16 + t] = (int)x.z; d[24 + t] = (int)x.w;
            d[4 + t] = (int)y.x; d[12 + t] = (int)y.y; d[20 + t] = (int)y.z; d[28 + t] = (int)y.w;
        } else {
            const u32x2 x = *(const u32x2 *)(uintptr_t)(a + (uint64_t)(SG.soa + t * nb + 4 * c));
            const u32x2 y = *(const u32x2 *)(uintptr_t)(b + (uint64_t)(SG.sob + t * nb + 4 * c));
            d[t] = (int)x.x; d[8 + t] = (int)x.y; d[4 + t] = (int)y.x; d[12 + t] = (int)y.y;
        }
    }
}
// The scale bytes of a product through LDS.  A wave's scale load from global memory touches 32
// cache lines (one row's 8 or 16 bytes out of each), and a chunk pair needs eight of them.  The
// scale rows of a region's 256 rows are one contiguous block of 256 * nb / 32 bytes per operand and
// product, which global -> LDS requests move in whole lines: four requests per wave and product
// (two per operand; a request beyond the block has a descriptor of length zero), issued a product
// ahead.  (Measured: 2 % of the run time of the MXFP8 and MXFP6 kernels, none of MXFP4's; all that
// the scale operands bring - loads, address arithmetic, shifts, registers - costs 7-12 %.)
template <int FMT>
__device__ __forceinline__ void big_request_scales(const BigSource &S, const BigScaleGeom &SG, int buf, int wave)
{
#pragma unroll
    for (int op = 0; op < 2; ++op)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int piece = wave * 2 + h;                  // 1 KB pieces of the operand's block
            const int block = 256 * SG.rb;
            const int bytes = (S.bytes != 0 && piece * 1024 < block) ? block : 0;
            big_dma_one((op ? S.b : S.a) + (uint64_t)(op ? SG.ub : SG.ua), bytes, SG.lane16, uni(piece * 1024),
                        (unsigned)uni(kBigLdsBytes + buf * kBigScaleBuf + op * kBigScaleOperand + piece * 1024));
        }
}
// The words big_load_scales delivers, read from scale buffer `buf` instead.
template <int FMT>
__device__ __forceinline__ void big_read_scales(int (&d)[32], const BigScaleGeom &SG, const char *lds, int buf, int c)
{
    c += SG.rot;
    if (c >= SG.n) c -= SG.n;
    const char *p = lds + kBigLdsBytes + buf * kBigScaleBuf;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        if constexpr (FMT == 2) {
            const u32x4 x = *(const u32x4 *)(p + SG.la + t * 32 * SG.rb + 8 * c);
            const u32x4 y = *(const u32x4 *)(p + SG.lb + t * 32 * SG.rb + 8 * c);
            d[t] = (int)x.x; d[8 + t] = (int)x.y; d[16 + t] = (int)x.z; d[24 + t] = (int)x.w;
            d[4 + t] = (int)y.x; d[12 + t] = (int)y.y; d[20 + t] = (int)y.z; d[28 + t] = (int)y.w;
        } else {
            const u32x2 x = *(const u32x2 *)(p + SG.la + t * 32 * SG.rb + 4 * c);
            const u32x2 y = *(const u32x2 *)(p + SG.lb + t * 32 * SG.rb + 4 * c);
            d[t] = (int)x.x; d[8 + t] = (int)x.y; d[4 + t] = (int)y.x; d[12 + t] = (int)y.y;
        }
    }
}
// The FP4 operand of reduction step j (0, 1) of a half: 16 of the fragment's 32 bytes.
__device__ __forceinline__ i8v big_fp4_operand(const i8v &f, int j)
{
    return j ? i8v{f[4], f[5], f[6], f[7], 0, 0, 0, 0} : i8v{f[0], f[1], f[2], f[3], 0, 0, 0, 0};
}

// FMT 3 (FP16) / 4 (BF16): reduction step w (0, 1) of a half on the 32x32x16 matrix instruction.  A
// lane's operand is 16 bytes = 8 elements of its row, the indices 8 (lane / 32) ... of the
// instruction's sixteen; which eight of the chunk row a lane holds is the same for A and B (the
// w-th 16 bytes of its fragment), and over a half every 16-byte piece of the 64 bytes is met once.
typedef _Float16 h8v __attribute__((ext_vector_type(8)));
typedef __bf16 bf8v __attribute__((ext_vector_type(8)));
template <int FMT>
__device__ __forceinline__ f16v big_mfma16(const i8v &a, const i8v &b, const f16v &c, int w)
{
    const i32x4 x = w ? i32x4{a[4], a[5], a[6], a[7]} : i32x4{a[0], a[1], a[2], a[3]};
    const i32x4 y = w ? i32x4{b[4], b[5], b[6], b[7]} : i32x4{b[0], b[1], b[2], b[3]};
    if constexpr (FMT == 3) return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(h8v, x), __builtin_bit_cast(h8v, y), c, 0, 0, 0);
    else return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf8v, x), __builtin_bit_cast(bf8v, y), c, 0, 0, 0);
}

// All 256 accumulator registers of a wave times a power of two.  The accumulators live in
// accumulation registers, which the vector ALU cannot address: every value takes the road
// read - multiply - write back through a vector register.  Left to itself the compiler sends all
// values down this road at once and spills eighty accumulators to make room (on every product,
// rescaled or not); the empty statements make each block of sixteen complete the round trip
// before the next one sets out.
__device__ __forceinline__ void big_rescale(f16v (&acc)[4][4], float ratio)
{
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
            f16v t = acc[mt][nt];
            asm volatile("" : "+v"(t));
#pragma unroll
            for (int v = 0; v < 16; ++v) t[v] = t[v] * ratio;
            asm volatile("" : "+v"(t));
            acc[mt][nt] = t;
            asm volatile("" : "+a"(acc[mt][nt]));
        }
}

// One chunk held in `STAGE`.  On entry f[0] holds the fragments of its first half; on exit
// those of the next chunk's first half.  S2: the chunk two ahead, requested into STAGE.
// FMT 2 (MXFP4): a half holds two reduction steps of 64 four-bit elements; the first step's MFMAs
// carry the half's other instructions, the second step's follow.
// FMT != 0: sc holds the block scales of a chunk pair (see big_load_scales), this chunk's from
// sc[SO] on; sa / sb are not used.  TAKE: `raw` are the scale words of the following pair, loaded
// by the caller just before this call: they are taken over (shifted into place, into `nx`) right
// behind the wait in the middle of the chunk, the one point where nothing else is in flight, so
// that no other wait for them is needed.
template <int STAGE, int FMT, bool TAKE, int SO, bool LS = false>
__device__ __forceinline__ void big_chunk(f16v (&acc)[4][4], typename BigFrag<FMT>::type (&f)[2][8], const BigGeom &BG, const char *lds, const BigSource &S2,
                                          int sa, int sb, const int (&sc)[32], int (&raw)[32], int (&nx)[32], const BigScaleGeom &SG,
                                          const BigScaleTake tk = BigScaleTake{0, 0})
{
    constexpr bool MX = FMT == 1 || FMT == 5;
    constexpr int EL = FMT == 5 ? 2 : 0;                     // element format of the instruction: e4m3, or e2m3
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
            if constexpr (FMT == 3 || FMT == 4) {
                acc[mt][nt] = big_mfma16<FMT>(f[0][mt], f[0][4 + nt], acc[mt][nt], 0);
                acc[mt][nt] = big_mfma16<FMT>(f[0][mt], f[0][4 + nt], acc[mt][nt], 1);
            } else if constexpr (FMT == 2) acc[mt][nt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(big_fp4_operand(f[0][mt], 0), big_fp4_operand(f[0][4 + nt], 0), acc[mt][nt], 4, 4, 0, sc[SO + mt], 0, sc[SO + 4 + nt]);
            else if constexpr (MX) acc[mt][nt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(big_operand(f[0][mt]), big_operand(f[0][4 + nt]), acc[mt][nt], EL, EL, 0, sc[SO + mt], 0, sc[SO + 4 + nt]);
            else acc[mt][nt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(f[0][mt], f[0][4 + nt], acc[mt][nt], 0, 0, 0, sa, 0, sb);
            SCHED_FENCE();
            const int k = mt * 4 + nt;                       // second half's fragments, 16 bytes per position: B first
            big_read_half<FMT>(f[1][((k >> 1) + 4) & 7], BG, lds, STAGE, 1, ((k >> 1) + 4) & 7, k & 1);
            SCHED_FENCE();
        }
    if constexpr (FMT == 2) {
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt)
                acc[mt][nt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(big_fp4_operand(f[0][mt], 1), big_fp4_operand(f[0][4 + nt], 1), acc[mt][nt], 4, 4, 2, sc[SO + mt], 2, sc[SO + 4 + nt]);
    }
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");         // the next chunk, requested a chunk ago, has landed
#endif
    __syncthreads();                                         // ... in every wave; and all are done reading this stage
    if constexpr (TAKE) {
        // from LDS: read here, behind the barrier that has just published them where they are a product's first
        if constexpr (LS) big_read_scales<FMT>(raw, SG, lds, tk.buf, tk.c);
#pragma unroll
        for (int t = 0; t < (FMT == 2 ? 32 : 16); ++t) nx[t] = (int)((uint32_t)raw[t] >> SG.shift);
#if defined(__HIP_DEVICE_COMPILE__)
#pragma unroll
        for (int t = 0; t < (FMT == 2 ? 32 : 16); t += 8)
            asm volatile("" : "+v"(nx[t]), "+v"(nx[t + 1]), "+v"(nx[t + 2]), "+v"(nx[t + 3]), "+v"(nx[t + 4]), "+v"(nx[t + 5]), "+v"(nx[t + 6]), "+v"(nx[t + 7]));
#endif
    }
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
            if constexpr (FMT == 3 || FMT == 4) {
                acc[mt][nt] = big_mfma16<FMT>(f[1][mt], f[1][4 + nt], acc[mt][nt], 0);
                acc[mt][nt] = big_mfma16<FMT>(f[1][mt], f[1][4 + nt], acc[mt][nt], 1);
            } else if constexpr (FMT == 2) acc[mt][nt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(big_fp4_operand(f[1][mt], 0), big_fp4_operand(f[1][4 + nt], 0), acc[mt][nt], 4, 4, 0, sc[SO + 8 + mt], 0, sc[SO + 12 + nt]);
            else if constexpr (MX) acc[mt][nt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(big_operand(f[1][mt]), big_operand(f[1][4 + nt]), acc[mt][nt], EL, EL, 2, sc[SO + mt], 2, sc[SO + 4 + nt]);
            else acc[mt][nt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(f[1][mt], f[1][4 + nt], acc[mt][nt], 0, 0, 0, sa, 0, sb);
            SCHED_FENCE();
            const int k = mt * 4 + nt;
            big_read_half<FMT>(f[0][((k >> 1) + 4) & 7], BG, lds, STAGE ^ 1, 0, ((k >> 1) + 4) & 7, k & 1);
            big_request<FMT>(S2, BG, STAGE, k);
            SCHED_FENCE();
        }
    if constexpr (FMT == 2) {
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt)
                acc[mt][nt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(big_fp4_operand(f[1][mt], 1), big_fp4_operand(f[1][4 + nt], 1), acc[mt][nt], 4, 4, 2, sc[SO + 8 + mt], 2, sc[SO + 12 + nt]);
    }
}

// MX: the operand tiles are MXFP8 (block scales behind the elements, no tile scale).  A lane's 32
// operand bytes of a 64-index step are then the 16 bytes at index 16 g of the step's first 32
// indices and the 16 bytes at 16 g of its second 32 (that is how the instruction pairs data
// with block scales), instead of 32 consecutive ones.
// FMT 2: MXFP4 tiles: half a byte per element, so a tile row is nb / 2 bytes and a chunk (128
// bytes of each row) 256 reduction indices; a lane's 16 bytes per reduction step are one block of
// 32 elements, scaled by that lane's own byte, and the fragment reads are those of FMT 1.
// FMT 5: MXFP6 tiles: 24 bytes per block of 32 six-bit elements; a chunk is a panel of 128 reduction
// indices, 96 bytes of each row, stored row after row with the four blocks of a row rotated by
// (row / 8) (see fp6_group_offset), and sits in LDS as it does in memory: rows of 96 bytes.  A
// lane's operand of a 64-index step is the block 32 (lane / 32) ... of the step, scaled by that
// lane's own byte (as for FMT 2); the rotation puts the blocks that 32 lanes read from 32
// consecutive rows on all 64 banks.
// LS (block-scaled formats, tile sizes up to 1024): the scale bytes travel through LDS.
template <int FMT, bool LS = false>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(1, 1)))
void gemm_mp_fp8_region_kernel(GemmArgs P, const WorkItem *__restrict__ items)
{
    static_assert(!LS || FMT == 1 || FMT == 2 || FMT == 5, "scale bytes exist in the block-scaled formats only");
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    const uint64_t itw = table_u64((const uint64_t *)items, blockIdx.x);
    const int tileC = (int)(uint32_t)itw;
    const ArgsPtr K0 = args();
    const int nb = K0->nb, kt = K0->kt_eff;
    constexpr bool MX = FMT == 1 || FMT == 2 || FMT == 5;
    constexpr int kChunkBytes = FMT == 5 ? 96 : kRowBytes;   // bytes of a tile row per chunk
    const int pitch = FMT == 5 ? (nb >> 2) * 3 : FMT == 2 ? nb / 2 : (FMT == 3 || FMT == 4) ? 2 * nb : nb;   // bytes of a tile row
    const int arow0 = (int)((itw >> 32) & 0xffffu) * kBigMacro, brow0 = (int)((itw >> 48) & 0xffffu) * kBigMacro;
    const ProductDesc *prod = K0->prod + (int64_t)tileC * K0->KT;

    BigGeom BG;
    {
        const int r = lane >> 3, slot = lane & 7;
        const int seg = slot ^ (r >> 1);                     // instruction 0; odd instructions: ^ 4
        BG.voff[0][0] = (arow0 + wave * 64 + r) * pitch + seg * 16;
        BG.voff[1][0] = (brow0 + wave * 64 + r) * pitch + seg * 16;
        BG.voff[0][1] = BG.voff[0][0] ^ 64;
        BG.voff[1][1] = BG.voff[1][0] ^ 64;
        BG.dst = (unsigned)uni(wave * (64 * kRowBytes));
        BG.rows8 = 8 * pitch;
        if constexpr (FMT == 5) {
            BG.voff[0][0] = arow0 * 96 + wave * 6144 + lane * 16;
            BG.voff[1][0] = brow0 * 96 + wave * 6144 + lane * 16;
            BG.dst = (unsigned)uni(wave * 6144);
            BG.rows8 = nb * 96;
        }
        BG.n = pitch / kChunkBytes;
        // Regions of one C tile run side by side on one XCD and would otherwise ask its L2 for the
        // same 128-byte column of every panel row at the same time; each starts its pass over a
        // product's chunks at its own (even) chunk instead.
        BG.rot = (2 * (int)((((itw >> 32) & 0xffffu) + ((itw >> 48) & 0xffffu)) & 3u)) % BG.n;
        const int i = lane & 31, g = lane >> 5, x = (i >> 1) & 7;
#pragma unroll
        for (int st = 0; st < 2; ++st)
#pragma unroll
            for (int hc = 0; hc < 2; ++hc)
#pragma unroll
                for (int w = 0; w < 2; ++w) {
                    const int slot_r = ((FMT == 1 || FMT == 2) ? 4 * hc + g + 2 * w : 4 * hc + 2 * g + w) ^ x;
                    BG.ra[st][hc][w] = st * kBigStage + (wm * 128 + i) * kRowBytes + slot_r * 16;
                    BG.rb[st][hc][w] = st * kBigStage + kBigOperand + (wn * 128 + i) * kRowBytes + slot_r * 16;
                    if constexpr (FMT == 5) {
                        const int pos = (2 * hc + g + (i >> 3)) & 3;
                        BG.ra[st][hc][w] = st * kBigStage + (wm * 128 + i) * 96 + pos * 24;
                        BG.rb[st][hc][w] = st * kBigStage + kBigOperand + (wn * 128 + i) * 96 + pos * 24;
                    }
                }
    }

    BigScaleGeom SG{};
    if constexpr (MX) {
        SG.soa = nb * pitch + (arow0 + wm * 128 + (lane & 31)) * (nb / 32);
        SG.sob = nb * pitch + (brow0 + wn * 128 + (lane & 31)) * (nb / 32);
        SG.shift = 8 * (lane >> 5);
        SG.rot = BG.rot;
        SG.n = BG.n;
        SG.rb = nb / 32;
        SG.ua = nb * pitch + arow0 * SG.rb;
        SG.ub = nb * pitch + brow0 * SG.rb;
        SG.la = (wm * 128 + (lane & 31)) * SG.rb;
        SG.lb = kBigScaleOperand + (wn * 128 + (lane & 31)) * SG.rb;
        SG.lane16 = lane * 16;
    }
    const int wave_u = uni(wave);

    f16v acc[4][4];
    const int n = pitch / kChunkBytes;                       // chunks per product: even (the host sees to that)
    const int tile_bytes = nb * pitch;

    // FP16 tiles carry a power-of-two scale each, so the terms of product L count in units of
    // 2^(eA + eB) of that product.  The one set of accumulators follows: at a product whose unit
    // differs it is multiplied by the ratio of the units (exact: a power of two, kept far from
    // the ends of FP32's range by the two bounds in the loop).  Where the units of the products
    // summed so far and the next one lie more than 2^64 apart, the reduction is cut there: the
    // sum so far leaves through the epilogue (alpha and beta applied, written to C), and the
    // rest of the reduction starts again from zero accumulators as a segment of its own whose
    // epilogue adds to what is there.  Every other format has one segment.
    int e_cur = 0, e_hi = 0, e_lo = 0;
    int L0 = 0;                                              // first product of the segment
    bool again = false;                                      // the region has been written before
    do {
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[mt][nt][v] = 0.0f;
        int L = L0;
        if (kt > 0) {
            if (L0 > 0) __syncthreads();                     // every wave has left the stages of the segment before
            const ConstQuad rec0 = (ConstQuad)(uintptr_t)(prod + L0);
            u32x4 lo = rec0[0], hi = rec0[1];
            BigSource S;
            S.a = (uint64_t)lo.x | ((uint64_t)lo.y << 32);
            S.b = (uint64_t)lo.z | ((uint64_t)lo.w << 32);
            S.bytes = tile_bytes;
            S.c = 0;
#pragma unroll
            for (int j = 0; j < 16; ++j) big_request<FMT>(S, BG, 0, j);
            if constexpr (LS) big_request_scales<FMT>(S, SG, 0, wave_u);      // the product's scale rows, buffer 0
            S.c = 1;
#pragma unroll
            for (int j = 0; j < 16; ++j) big_request<FMT>(S, BG, 1, j);
#if defined(__HIP_DEVICE_COMPILE__)
            if constexpr (FMT == 5) asm volatile("s_waitcnt vmcnt(12)" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(16)" ::: "memory");    // chunk 0 has landed
#endif
            __syncthreads();
            typename BigFrag<FMT>::type f[2][8];
#pragma unroll
            for (int t = 0; t < 8; ++t) f[0][t] = big_read<FMT>(BG, lds, 0, 0, t);
            int sc[32], nsc[32];
#pragma unroll
            for (int t = 0; t < 32; ++t) sc[t] = nsc[t] = 0;
            if constexpr (MX) {
                big_load_scales<FMT>(sc, SG, S.a, S.b, nb, 0);
#pragma unroll
                for (int t = 0; t < 32; ++t) sc[t] = (int)((uint32_t)sc[t] >> SG.shift);
            }

            int sbuf = 0;                                    // scale buffer of the product being computed
            for (; L < kt; ++L) {
                int sa, sb;
                big_scales((int)hi.x, (int)hi.y, sa, sb);
                if constexpr (FMT == 3) {
                    const int e = (int)hi.x + (int)hi.y;
                    if (L == L0) {
                        e_cur = e_hi = e_lo = e;
                    } else if (e != e_cur) {
                        if (e_hi - e > 64 || e - e_lo > 64) break;       // cut the reduction here
                        const float ratio = __uint_as_float((uint32_t)(e_cur - e + 127) << 23);      // 2^(e_cur - e), |e_cur - e| <= 64
                        big_rescale(acc, ratio);
                        e_hi = e > e_hi ? e : e_hi;
                        e_lo = e < e_lo ? e : e_lo;
                        e_cur = e;
                    }
                }
                // the following product (descriptors of length zero past the end)
                u32x4 nlo = lo, nhi = hi;
                int nbytes = 0;
                if (L + 1 < kt) {
                    const ConstQuad rec = (ConstQuad)(uintptr_t)(prod + L + 1);
                    nlo = rec[0];
                    nhi = rec[1];
                    nbytes = tile_bytes;
                }
                BigSource cur_src, next_src;
                cur_src.a = (uint64_t)lo.x | ((uint64_t)lo.y << 32);
                cur_src.b = (uint64_t)lo.z | ((uint64_t)lo.w << 32);
                cur_src.bytes = tile_bytes;
                next_src.a = (uint64_t)nlo.x | ((uint64_t)nlo.y << 32);
                next_src.b = (uint64_t)nlo.z | ((uint64_t)nlo.w << 32);
                next_src.bytes = nbytes;
                // The following product's scale rows go to the other scale buffer.  No wave reads that
                // buffer any more: it held the scales of the product before this one, last read in the
                // middle of that product's last chunk pair but one, at least two barriers ago (the last
                // pair of a product takes over the first scales of the next, from this product's buffer).
                if constexpr (LS) big_request_scales<FMT>(next_src, SG, sbuf ^ 1, wave_u);
                for (int c = 0; c < n; c += 2) {
                    BigSource S2 = (c + 2 < n) ? cur_src : next_src;
                    S2.c = (c + 2 < n) ? c + 2 : c + 2 - n;
                    // block scales of what follows are fetched under the chunk being computed (past the
                    // end of the reduction: those of the last chunks again, unused)
                    int nx[32];
#pragma unroll
                    for (int t = 0; t < 32; ++t) nx[t] = 0;
                    if constexpr (MX) {
                        // sc holds the scales of chunks c and c + 1; those of the next pair are requested
                        // before the second chunk and taken over in its middle
                        const bool wrap = c + 2 >= n && nbytes != 0;
                        const int cnext = c + 2 < n ? c + 2 : wrap ? 0 : n - 2;
                        big_chunk<0, FMT, false, 0>(acc, f, BG, lds, S2, sa, sb, sc, nsc, nx, SG);
                        if constexpr (!LS)
                            big_load_scales<FMT>(nsc, SG, wrap ? next_src.a : cur_src.a, wrap ? next_src.b : cur_src.b, nb, cnext);
                        S2.c += 1;
                        big_chunk<1, FMT, true, FMT == 2 ? 16 : 8, LS>(acc, f, BG, lds, S2, sa, sb, sc, nsc, nx, SG,
                                                                       BigScaleTake{wrap ? sbuf ^ 1 : sbuf, cnext});
#pragma unroll
                        for (int t = 0; t < 32; ++t) sc[t] = nx[t];
                    } else {
                        big_chunk<0, FMT, false, 0>(acc, f, BG, lds, S2, sa, sb, sc, nsc, nx, SG);
                        S2.c += 1;
                        big_chunk<1, FMT, false, 0>(acc, f, BG, lds, S2, sa, sb, sc, nsc, nx, SG);
                    }
                }
                lo = nlo;
                hi = nhi;
                sbuf ^= 1;
            }
#if defined(__HIP_DEVICE_COMPILE__)
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // requests past the segment's end still write into the stages
#endif
        }

        // Epilogue: v = alpha*s (+ beta*c0), two rounded products and one rounded sum in FP32.  A
        // 32 x 32 accumulator block holds, per register, one row piece of 32 consecutive columns
        // in each half of the wave: 128-byte row segments straight from the registers.  FP16
        // tiles: the accumulators hold the sum in units of 2^e_cur.  A later segment adds to what
        // the earlier ones wrote (beta has been applied by the first).
        const ArgsPtr K = args();
        const float alpha = (float)K->alpha, beta = again ? 1.0f : (float)K->beta;
        const bool use_c = again || K->beta != 0.0;
        typedef __attribute__((address_space(1))) float *GlobalF;
        GlobalF ctile = (GlobalF)(uintptr_t)(K->C.storage + table_u64(K->C.offset, tileC));
        GlobalF cbase = ctile + (int64_t)(arow0 + wm * 128 + 4 * (lane >> 5)) * nb + brow0 + wn * 128 + (lane & 31);
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) {
                float c0[16];
                if (use_c) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) c0[v] = cbase[(int64_t)(mt * 32 + 8 * (v >> 2) + (v & 3)) * nb + nt * 32];
                }
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    float val = alpha * (FMT == 3 ? ldexpf(acc[mt][nt][v], e_cur) : acc[mt][nt][v]);
                    if (use_c) { const float bc = beta * c0[v]; val = val + bc; }
                    // a streaming store: the C block is written once and not read again, and it must
                    // not push the operand panels, which fifteen other regions are reading, out of L2
#ifdef GMP_PLAIN_C_STORES                              /* a build switch for comparisons only */
                    cbase[(int64_t)(mt * 32 + 8 * (v >> 2) + (v & 3)) * nb + nt * 32] = val;
#else
                    __builtin_nontemporal_store(val, &cbase[(int64_t)(mt * 32 + 8 * (v >> 2) + (v & 3)) * nb + nt * 32]);
#endif
                }
            }
        again = true;
        L0 = L;
    } while (FMT == 3 && L0 < kt);
}

}  // namespace gmp

#define GMP_REGION_INSTANCE(NAME, FMT)                                                                      \
    namespace gmp {                                                                                         \
    constexpr bool kScaled_##NAME = (FMT) == 1 || (FMT) == 2 || (FMT) == 5;                                 \
    hipError_t setup_##NAME()                                                                               \
    {                                                                                                       \
        hipError_t e = hipFuncSetAttribute((const void *)gemm_mp_fp8_region_kernel<FMT, false>,             \
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kBigLdsBytes);       \
        if (e != hipSuccess || !kScaled_##NAME) return e;                                                   \
        return hipFuncSetAttribute((const void *)gemm_mp_fp8_region_kernel<FMT, kScaled_##NAME>,            \
                                   hipFuncAttributeMaxDynamicSharedMemorySize, kBigLdsScaled);              \
    }                                                                                                       \
    hipError_t launch_##NAME(const GemmArgs &a, const WorkItem *items, int n, hipStream_t s)                \
    {                                                                                                       \
        /* block-scaled tiles of up to 1024: the instance that moves the scale bytes through LDS */         \
        if (kScaled_##NAME && a.nb <= 1024)                                                                 \
            gemm_mp_fp8_region_kernel<FMT, kScaled_##NAME><<<dim3((unsigned)n), dim3(kThreads), kBigLdsScaled, s>>>(a, items); \
        else                                                                                                \
            gemm_mp_fp8_region_kernel<FMT, false><<<dim3((unsigned)n), dim3(kThreads), kBigLdsBytes, s>>>(a, items); \
        return hipGetLastError();                                                                           \
    }                                                                                                       \
    }
