// Internal declarations shared by the host side of the library and its HIP kernels.
#pragma once
#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>

#include "../../include/gemm_mp.h"

namespace gmp {

constexpr int kMacro = 128;       // rows = cols of C owned by one workgroup
constexpr int kMacroFp8 = 256;    // the same for C tiles whose products are all FP8 x FP8
constexpr int kScanCols = 128;    // columns one scan workgroup reduces; a power of two
constexpr int kPackBlock = 64;    // pack / unpack move 64 x 64 element blocks
constexpr int kConvSlots = 8;     // sender-side copies of a tile: one slot per product precision code (0..4 used)
constexpr int kLowChunk = 4096;   // elements one workgroup handles in the passes over FP16 / FP8 C tiles

// Bytes per element of each precision code.
__host__ __device__ inline int elem_bytes(int p) { return p == 0 ? 8 : p == 1 ? 4 : (p == 2 || p == 4) ? 2 : 1; }
// Bytes of a packed tile of nb x nb elements (block-scaled tiles: elements, then one scale byte per 32).
__host__ __device__ inline uint64_t tile_bytes_of(int p, uint64_t elems)
{
    if (p == GEMM_MP_MXFP8) return elems + elems / 32;
    if (p == GEMM_MP_MXFP4) return elems / 2 + elems / 32;
    if (p == GEMM_MP_MXFP6) return elems / 4 * 3 + elems / 32;
    return elems * (uint64_t)elem_bytes(p);
}
__host__ __device__ inline bool is_block_scaled(int p) { return p == GEMM_MP_MXFP8 || p == GEMM_MP_MXFP4 || p == GEMM_MP_MXFP6; }

// Value of a six-bit e2m3 code: sign, two exponent bits (bias 1), three fraction bits; exact in FP32.
__host__ __device__ inline float fp6_value(uint32_t code)
{
    const int ef = (int)(code >> 3) & 3, mf = (int)code & 7;
    const float mag = ef ? (float)((8 + mf) << (ef - 1)) * 0.125f : 0.125f * (float)mf;
    return (code & 32u) ? -mag : mag;
}

// Where the six-bit codes of an MXFP6 tile lie.  The elements of a tile are stored panel by panel:
// a panel holds 128 consecutive reduction indices (four blocks of 32; tile sizes are multiples of
// 128) of every packed row, row after row, 96 bytes each, so that the part of a
// panel that 256 rows take up is one contiguous piece of memory which the 256 x 256 kernel copies to
// LDS as it is.  Inside a row of a panel the blocks are rotated by (row / 8): block b sits at block
// position (b + row / 8) mod 4, which spreads the block that 32 lanes read from 32 consecutive rows
// over all LDS banks.  Returned: the byte offset, from the start of the tile, of the three bytes
// that hold the elements k .. k + 3 (k a multiple of 4) of packed row r.
__host__ __device__ inline int64_t fp6_group_offset(int nb, int r, int k)
{
    const int pos = (((k >> 5) & 3) + (r >> 3)) & 3;
    return (int64_t)(k >> 7) * nb * 96 + (int64_t)r * 96 + pos * 24 + ((k & 31) >> 2) * 3;
}

// Product precision (code) for stored precisions pA, pB, C tile precision pC.
__host__ __device__ inline int product_precision(int pA, int pB, int pC, int policy)
{
    const int cap = (pC == GEMM_MP_FP64) ? GEMM_MP_FP64 : GEMM_MP_FP32;
    if (policy == GEMM_MP_POLICY_C_TILE) return cap;
    // the smallest format that holds both operands' numbers: FP64 > FP32 > {FP16, BF16} > FP8
    if (pA == GEMM_MP_MXFP8 && pB == GEMM_MP_MXFP8) return GEMM_MP_MXFP8;
    if (pA == GEMM_MP_MXFP4 && pB == GEMM_MP_MXFP4) return GEMM_MP_MXFP4;
    if (pA == GEMM_MP_MXFP6 && pB == GEMM_MP_MXFP6) return GEMM_MP_MXFP6;
    if (is_block_scaled(pA)) pA = GEMM_MP_FP32;                             // block-scaled numbers are FP32 numbers
    if (is_block_scaled(pB)) pB = GEMM_MP_FP32;
    int q;
    const bool h = pA == GEMM_MP_FP16 || pB == GEMM_MP_FP16, b = pA == GEMM_MP_BF16 || pB == GEMM_MP_BF16;
    if (pA == GEMM_MP_FP64 || pB == GEMM_MP_FP64) q = GEMM_MP_FP64;
    else if (pA == GEMM_MP_FP32 || pB == GEMM_MP_FP32 || (h && b)) q = GEMM_MP_FP32;
    else q = h ? GEMM_MP_FP16 : b ? GEMM_MP_BF16 : GEMM_MP_FP8_E4M3;
    return (q == GEMM_MP_FP64 && cap == GEMM_MP_FP32) ? GEMM_MP_FP32 : q;
}

// Device-side view of one packed matrix.
struct PackedView {
    const uint8_t *prec;     // [tiles] precision code
    const uint64_t *offset;  // [tiles] byte offset into storage
    const int32_t *exp;      // [tiles] power-of-two scale exponent
    char *storage;
};

// One owner workgroup: C tile index and the macro-tile inside it.
struct WorkItem {
    uint32_t tile;   // I * NT + J
    uint16_t mi, mj; // macro-tile row / column inside the tile
};

// Everything the GEMM kernel needs to know about one tile product A(I,L)*B(L,J), gathered into
// one 32-byte record so that a workgroup opens a product with a single scalar load.  The table
// is [MT*NT][KT] (C tile major) and is rebuilt on the device before every run from the maps,
// offsets and exponents current at that time.
struct ProductDesc {
    uint64_t a_ptr, b_ptr;   // device addresses of the two operand tiles (packed storage, or the
                             // sender-side workspace when a converted copy exists)
    int32_t ea, eb;          // their scale exponents
    uint32_t codes;          // pA | pB << 8 | q << 16, pA / pB as the kernel finds them there; BF16 is
                             // written as FP16 (the same element size) with a flag: bit 24 A, 25 B, 26 q
    uint32_t pad;
};

// One sender-side conversion: tile `tile` of a packed matrix (precision p at src) to precision
// q at dst; n16 = number of 16-byte segments of the result.
struct ConvertJob {
    uint64_t src, dst;
    uint32_t tile;           // index into the matrix's exponent table
    uint8_t p, q, which, pad;
    uint32_t n16;
    uint32_t nb;             // tile size (the layout of an MXFP6 source depends on it)
};

// A C tile stored in FP16 / FP8: its index and the byte offset, in C's buffer, of the FP32
// staging copy the GEMM kernels accumulate into.
struct LowTile {
    uint64_t stage;
    uint32_t tile;
    uint32_t pad;
};

static_assert(sizeof(ProductDesc) == 32, "the kernel reads a record as two 16-byte scalar loads");
static_assert(sizeof(WorkItem) == 8, "the kernel reads an item as one 8-byte scalar load");

struct GemmArgs {
    PackedView A, B, C;
    const uint8_t *q;        // [MT*NT][KT] product precision of every task
    ProductDesc *prod;       // [MT*NT][KT] (+ padding records), written by launch_gemm
    const uint64_t *convA;   // [tiles of A][kConvSlots] address of the copy converted to q, 0 = none; or null
    const uint64_t *convB;   // same for B
    const WorkItem *items64;  // owner regions of FP64 C tiles, launch order
    const WorkItem *items32;  // owner regions of FP32 C tiles, launch order
    const WorkItem *items8;   // 256 x 256 regions of FP32 C tiles made of FP8 x FP8 products only
    const WorkItem *items_mx; // the same of tiles made of MXFP8 x MXFP8 products only
    const WorkItem *items_mx4;// ... of MXFP4 x MXFP4 products only
    const WorkItem *items_h;  // ... of FP16 x FP16 products only
    const WorkItem *items_bf; // ... of BF16 x BF16 products only
    const WorkItem *items_mx6;// ... of MXFP6 x MXFP6 products only
    int32_t n_items64, n_items32, n_items8, n_items_mx, n_items_mx4, n_items_h, n_items_bf, n_items_mx6;
    int32_t mixed32;         // some region of items32 has an FP16 / BF16 product with an operand stored in FP8
    int32_t mixed64;         // the same for items64
    int32_t low64;           // no region of items64 has an FP64 product
    int32_t bf16;            // some product of the 128 x 128 kernels has a BF16 or block-scaled operand
    int32_t nb, MT, NT, KT;
    int32_t kt_eff;          // KT, or 0 when alpha == 0
    double alpha, beta;
};

// rows x cols: the entries the dense matrix has; rows_t x cols_t: its tiles (the last ones may
// stick out over the edge and are zero-padded).
hipError_t launch_scan(const double *X, int64_t ld, bool transposed, int64_t rows, int64_t cols, int rows_t, int cols_t, int nb,
                       double *part_sum, double *part_max, double *sumsq, double *maxabs,
                       hipStream_t s);
hipError_t launch_exps(const double *maxabs, const uint8_t *prec, int32_t *exps, int ntiles,
                       hipStream_t s);
hipError_t launch_pack(const double *X, int64_t ld, int64_t rows, int64_t cols, int rows_t, int cols_t, int nb, bool turn,
                       bool swap, PackedView v, hipStream_t s);
// MXFP8 tiles of a matrix: block quantisation along the reduction index (is_b: down the columns).
// Entry (r, c) of the matrix is X[r * sr + c * sc].
hipError_t launch_pack_mx(const double *X, int64_t sr, int64_t sc, int64_t rows, int64_t cols, int rows_t, int cols_t, int nb,
                          bool is_b, PackedView v, hipStream_t s);
hipError_t launch_unpack(double *X, int64_t ld, int64_t rows, int64_t cols, int rows_t, int cols_t, int nb, bool turn,
                         bool swap, PackedView v, hipStream_t s);
// Side streams (default priority) and events for running the launches of one gemm_mp_run side by side.
struct LaunchLanes {
    hipStream_t side[4];
    hipEvent_t fork;
    hipEvent_t join[4];
};
hipError_t launch_gemm(const GemmArgs &a, hipStream_t s, const LaunchLanes *lanes);
hipError_t launch_convert(const ConvertJob *jobs_dev, int njobs, uint32_t max_n16, const int32_t *expA, const int32_t *expB,
                          hipStream_t s);
hipError_t launch_low_expand(const LowTile *low_dev, int n_low, int nb, PackedView c, hipStream_t s);
hipError_t launch_low_store(const LowTile *low_dev, int n_low, int nb, PackedView c, int32_t *exps, float *part_max,
                            hipStream_t s);
hipError_t gemm_kernel_setup();
// One pair per kernel instance, each defined in its own translation unit (gemm_<name>.hip).
#define GMP_DECLARE_INSTANCE(NAME) \
    hipError_t setup_##NAME();     \
    hipError_t launch_##NAME(const GemmArgs &a, const WorkItem *items, int n, hipStream_t s);
GMP_DECLARE_INSTANCE(owner_d) GMP_DECLARE_INSTANCE(owner_d_mixed) GMP_DECLARE_INSTANCE(owner_d_bf) GMP_DECLARE_INSTANCE(owner_d_low)
GMP_DECLARE_INSTANCE(owner_f) GMP_DECLARE_INSTANCE(owner_f_mixed) GMP_DECLARE_INSTANCE(owner_f_bf)
GMP_DECLARE_INSTANCE(region_fp8) GMP_DECLARE_INSTANCE(region_mxfp8) GMP_DECLARE_INSTANCE(region_mxfp4)
GMP_DECLARE_INSTANCE(region_fp16) GMP_DECLARE_INSTANCE(region_bf16) GMP_DECLARE_INSTANCE(region_mxfp6)

}  // namespace gmp
