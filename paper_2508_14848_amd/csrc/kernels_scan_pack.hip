// Tile scan, pack (storage rounding + re-tiling) and unpack kernels for gfx950.
// All three are HBM-bound streaming passes over a dense row-major FP64 matrix.
#include "gemm_mp_internal.h"

namespace gmp {

// ---------------------------------------------------------------------------------------
// Tile scan.  One thread owns one column of one tile row and walks down its nb rows with a
// running fused multiply-add (the defined order of the tile's sum of squares); a wave reads
// 512 contiguous bytes per row.  The 128 column sums of a workgroup are then added pairwise,
// neighbours first; because nb is a multiple of 128 these seven levels are exactly the lowest
// seven levels of the pairing over the whole tile.  scan_finish_kernel adds the nb/128 roots
// of a tile with the same rule (an odd element is carried up).  The matrix has rows x cols
// entries; a tile that sticks out over its edge counts the missing entries as zeros (adding
// fma(0, 0, s) leaves s as it is, so the sums are those of the zero-padded matrix bit for bit).
// Entry (r, c) of the matrix is X[r * sr + c * sc]: (ld, 1) as given, (1, ld) when the buffer
// holds the transpose; the order of the sums is that of the matrix, not of the buffer.
__global__ __launch_bounds__(kScanCols) void scan_cols_kernel(const double *__restrict__ X,
                                                              int64_t sr, int64_t sc, int64_t rows, int64_t cols, int nb, int parts,
                                                              int cols_t,
                                                              double *__restrict__ part_sum,
                                                              double *__restrict__ part_max)
{
    __shared__ double vs[kScanCols];
    __shared__ double vm[kScanCols];
    const int tx = threadIdx.x;
    const int64_t col = (int64_t)blockIdx.x * kScanCols + tx;
    const int I = blockIdx.y;
    const double *p = X + (int64_t)I * nb * sr + col * sc;
    double s = 0.0, m = 0.0;
    const int64_t left = rows - (int64_t)I * nb;                 // rows of the matrix from this tile row on
    const int rmax = col < cols ? (left < nb ? (int)left : nb) : 0;
    int r = 0;
    for (; r + 8 <= rmax; r += 8) {
        double x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) x[u] = p[(int64_t)(r + u) * sr];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            s = __builtin_fma(x[u], x[u], s);
            const double ax = __builtin_fabs(x[u]);
            if (ax > m) m = ax;      // a NaN never enters m
        }
    }
    for (; r < rmax; ++r) {          // the last rows of a matrix whose row count is no multiple of 8
        const double x = p[(int64_t)r * sr];
        s = __builtin_fma(x, x, s);
        const double ax = __builtin_fabs(x);
        if (ax > m) m = ax;
    }
    vs[tx] = s;
    vm[tx] = m;
    __syncthreads();
    for (int n = kScanCols / 2; n >= 1; n >>= 1) {
        double a = 0.0, b = 0.0;
        if (tx < n) {
            a = vs[2 * tx] + vs[2 * tx + 1];
            const double m0 = vm[2 * tx], m1 = vm[2 * tx + 1];
            b = m1 > m0 ? m1 : m0;
        }
        __syncthreads();
        if (tx < n) { vs[tx] = a; vm[tx] = b; }
        __syncthreads();
    }
    if (tx == 0) {
        const int J = (int)((int64_t)blockIdx.x * kScanCols / nb);
        const int part = (int)(((int64_t)blockIdx.x * kScanCols % nb) / kScanCols);
        const int64_t o = ((int64_t)I * cols_t + J) * parts + part;
        part_sum[o] = vs[0];
        part_max[o] = vm[0];
    }
}

__global__ void scan_finish_kernel(const double *__restrict__ part_sum,
                                   const double *__restrict__ part_max, int parts, int ntiles,
                                   double *__restrict__ sumsq, double *__restrict__ maxabs)
{
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= ntiles) return;
    double v[64];
    double m = 0.0;
    int n = parts;
    for (int i = 0; i < n; ++i) {
        v[i] = part_sum[(int64_t)t * parts + i];
        const double x = part_max[(int64_t)t * parts + i];
        if (x > m) m = x;
    }
    while (n > 1) {
        const int h = n / 2;
        for (int i = 0; i < h; ++i) v[i] = v[2 * i] + v[2 * i + 1];
        if (n & 1) { v[h] = v[n - 1]; n = h + 1; } else n = h;
    }
    sumsq[t] = v[0];
    maxabs[t] = m;
}

hipError_t launch_scan(const double *X, int64_t ld, bool transposed, int64_t rows, int64_t cols, int rows_t, int cols_t, int nb,
                       double *part_sum, double *part_max, double *sumsq, double *maxabs,
                       hipStream_t s)
{
    const int parts = nb / kScanCols;
    dim3 grid((unsigned)((int64_t)cols_t * nb / kScanCols), (unsigned)rows_t);
    scan_cols_kernel<<<grid, kScanCols, 0, s>>>(X, transposed ? 1 : ld, transposed ? ld : 1, rows, cols, nb, parts, cols_t,
                                                part_sum, part_max);
    const int ntiles = rows_t * cols_t;
    scan_finish_kernel<<<(ntiles + 63) / 64, 64, 0, s>>>(part_sum, part_max, parts, ntiles, sumsq, maxabs);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Scale exponent of FP16 / FP8 tiles: e = floor(log2 max|x|) - 14 (FP16) or - 7 (FP8), so the
// largest scaled magnitude lies in [2^14,2^15) resp. [2^7,2^8); 0 for an all-zero tile, a
// non-finite maximum, and for FP64 / FP32 tiles.  floor(log2) is read off the bit pattern.
__global__ void exps_kernel(const double *__restrict__ maxabs, const uint8_t *__restrict__ prec,
                            int32_t *__restrict__ exps, int ntiles)
{
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= ntiles) return;
    const int p = prec[t];
    int e = 0;
    if (p == GEMM_MP_FP16 || p == GEMM_MP_FP8_E4M3) {
        const uint64_t bits = (uint64_t)__double_as_longlong(maxabs[t]) & 0x7fffffffffffffffull;
        const int field = (int)(bits >> 52);
        const uint64_t man = bits & 0xfffffffffffffull;
        if (field == 0x7ff || bits == 0) e = 0;
        else {
            const int lg = field ? field - 1023 : 63 - __builtin_clzll(man) - 1074;
            e = lg - (p == GEMM_MP_FP16 ? 14 : 7);
        }
    }
    exps[t] = e;
}

hipError_t launch_exps(const double *maxabs, const uint8_t *prec, int32_t *exps, int ntiles,
                       hipStream_t s)
{
    exps_kernel<<<(ntiles + 63) / 64, 64, 0, s>>>(maxabs, prec, exps, ntiles);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Storage rounding of x * 2^-e from FP64 into a small binary format, one rounding to nearest
// even, done on the bit pattern.  MB fraction bits, EMIN exponent of the smallest normal, BIAS.
// Returns the magnitude code (sign not included), before any overflow treatment; the exponent
// field may exceed the format's range, which the callers turn into infinity / saturation.
template <int MB, int EMIN, int BIAS>
__device__ inline uint32_t round_magnitude(uint64_t mag_bits, int e)
{
    const int field = (int)(mag_bits >> 52);
    uint64_t sig = mag_bits & 0xfffffffffffffull;
    int E;                                                     // exponent of x * 2^-e
    if (field) { sig |= 1ull << 52; E = field - 1023 - e; }
    else {
        if (sig == 0) return 0;
        const int lz = __builtin_clzll(sig) - 11;              // FP64 subnormal: normalise first
        sig <<= lz;
        E = -1022 - lz - e;
    }
    int drop = 52 - MB;                                        // low bits that do not fit
    if (E < EMIN) drop += EMIN - E;                            // subnormal range: coarser grid
    if (drop >= 55) return 0;                                  // below a quarter of the smallest step
    uint64_t kept = sig >> drop;
    const uint64_t rem = sig & ((1ull << drop) - 1);
    const uint64_t half = 1ull << (drop - 1);
    if (rem > half || (rem == half && (kept & 1))) ++kept;     // nearest, ties to even
    if (E < EMIN) return (uint32_t)kept;                       // exponent field 0 (or 1 after a carry)
    if (E > 4096) return 0x7fffffffu;                          // keeps the shift below in range
    return (uint32_t)(((uint64_t)(E + BIAS) << MB) + (kept - (1ull << MB)));   // a carry bumps the exponent
}

__device__ inline uint32_t to_fp16_bits(double x, int e)
{
    const uint64_t b = (uint64_t)__double_as_longlong(x);
    const uint32_t sign = (uint32_t)(b >> 48) & 0x8000u;
    const uint64_t mag = b & 0x7fffffffffffffffull;
    if (mag > 0x7ff0000000000000ull) return sign | 0x7e00u;    // NaN
    if (mag == 0x7ff0000000000000ull) return sign | 0x7c00u;   // infinity
    uint32_t r = round_magnitude<10, -14, 15>(mag, e);
    if (r > 0x7c00u) r = 0x7c00u;                              // overflow -> infinity
    return sign | r;
}

__device__ inline uint32_t to_fp8_bits(double x, int e)
{
    const uint64_t b = (uint64_t)__double_as_longlong(x);
    const uint32_t sign = (uint32_t)(b >> 56) & 0x80u;
    const uint64_t mag = b & 0x7fffffffffffffffull;
    if (mag > 0x7ff0000000000000ull) return sign | 0x7fu;      // NaN
    if (mag == 0x7ff0000000000000ull) return sign | 0x7eu;     // no infinity: saturate
    uint32_t r = round_magnitude<3, -6, 7>(mag, e);
    if (r > 0x7eu) r = 0x7eu;                                  // beyond 448 -> 448
    return sign | r;
}

// BF16 has FP32's exponent range: no tile scale, overflow to infinity.
__device__ inline uint32_t to_bf16_bits(double x)
{
    const uint64_t b = (uint64_t)__double_as_longlong(x);
    const uint32_t sign = (uint32_t)(b >> 48) & 0x8000u;
    const uint64_t mag = b & 0x7fffffffffffffffull;
    if (mag > 0x7ff0000000000000ull) return sign | 0x7fc0u;    // NaN
    if (mag == 0x7ff0000000000000ull) return sign | 0x7f80u;   // infinity
    uint32_t r = round_magnitude<7, -126, 127>(mag, 0);
    if (r > 0x7f80u) r = 0x7f80u;                              // overflow -> infinity
    return sign | r;
}

// FP4 e2m1 (1 fraction bit, smallest normal 1, largest 6; no infinity or NaN codes: both
// saturate resp. become 0), after scaling by 2^-e.
__device__ inline uint32_t to_fp4_bits(double x, int e)
{
    const uint64_t b = (uint64_t)__double_as_longlong(x);
    const uint32_t sign = (uint32_t)(b >> 60) & 0x8u;
    const uint64_t mag = b & 0x7fffffffffffffffull;
    if (mag > 0x7ff0000000000000ull) return 0;                 // NaN has no code
    if (mag == 0x7ff0000000000000ull) return sign | 7u;
    uint32_t r = round_magnitude<1, 0, 1>(mag, e);
    if (r > 7u) r = 7u;                                        // beyond 6 -> 6
    return r ? (sign | r) : sign;
}

// FP6 e2m3 (3 fraction bits, smallest normal 1, largest 7.5; no infinity or NaN codes, as FP4).
__device__ inline uint32_t to_fp6_bits(double x, int e)
{
    const uint64_t b = (uint64_t)__double_as_longlong(x);
    const uint32_t sign = (uint32_t)(b >> 58) & 0x20u;
    const uint64_t mag = b & 0x7fffffffffffffffull;
    if (mag > 0x7ff0000000000000ull) return 0;                 // NaN has no code
    if (mag == 0x7ff0000000000000ull) return sign | 31u;
    uint32_t r = round_magnitude<3, 0, 1>(mag, e);
    if (r > 31u) r = 31u;                                      // beyond 7.5 -> 7.5
    return sign | r;
}
// The stored bit pattern of one element, right-aligned in 64 bits.
__device__ inline uint64_t stored_bits(double x, int p, int e)
{
    switch (p) {
    case GEMM_MP_FP64: return (uint64_t)__double_as_longlong(x);
    case GEMM_MP_FP32: return (uint64_t)__float_as_uint((float)x);     // v_cvt_f32_f64, nearest even
    case GEMM_MP_FP16: return to_fp16_bits(x, e);
    case GEMM_MP_BF16: return to_bf16_bits(x);
    default:           return to_fp8_bits(x, e);
    }
}

__device__ inline void store4(char *dst, int p, const uint64_t (&v)[4])
{
    switch (p) {
    case GEMM_MP_FP64: {
        ulonglong2 a, b;
        a.x = v[0]; a.y = v[1]; b.x = v[2]; b.y = v[3];
        ((ulonglong2 *)dst)[0] = a;
        ((ulonglong2 *)dst)[1] = b;
    } break;
    case GEMM_MP_FP32: {
        uint4 a;
        a.x = (uint32_t)v[0]; a.y = (uint32_t)v[1]; a.z = (uint32_t)v[2]; a.w = (uint32_t)v[3];
        *(uint4 *)dst = a;
    } break;
    case GEMM_MP_FP16:
    case GEMM_MP_BF16: {
        uint2 a;
        a.x = (uint32_t)v[0] | ((uint32_t)v[1] << 16);
        a.y = (uint32_t)v[2] | ((uint32_t)v[3] << 16);
        *(uint2 *)dst = a;
    } break;
    default:
        *(uint32_t *)dst = (uint32_t)v[0] | ((uint32_t)v[1] << 8) | ((uint32_t)v[2] << 16) | ((uint32_t)v[3] << 24);
    }
}

// Pack: each workgroup converts one 64 x 64 block that lies inside one tile.  Threads read four
// consecutive FP64 values of a row (coalesced 512 B per 16 lanes); for A and C they store the
// four converted values directly; for B the block is turned through LDS so that the stores run
// along the reduction index, which is the contiguous one in a packed B tile.  A block on the
// edge of a rows x cols matrix reads only what exists and stores zeros for the rest, so every
// packed tile is a full tile of the zero-padded matrix.
template <bool TRANSPOSE>
__global__ __launch_bounds__(256) void pack_kernel(const double *__restrict__ X, int64_t ld, int64_t rows, int64_t cols, int nb,
                                                   int rows_t, int cols_t, bool swap, PackedView v)
{
    __shared__ uint64_t turn[TRANSPOSE ? kPackBlock : 1][TRANSPOSE ? kPackBlock + 1 : 1];
    const int t = threadIdx.x;
    const int64_t R0 = (int64_t)blockIdx.y * kPackBlock, C0 = (int64_t)blockIdx.x * kPackBlock;
    const int I = (int)(R0 / nb), J = (int)(C0 / nb);
    const int tile = swap ? J * rows_t + I : I * cols_t + J;      // swap: the buffer holds the matrix's transpose
    const int p = v.prec[tile];
    if (is_block_scaled(p)) return;                              // block-scaled tiles: pack_mx_kernel
    const int e = v.exp[tile];
    char *base = v.storage + v.offset[tile];
    const int r_in = (int)(R0 % nb), c_in = (int)(C0 % nb);
    const int es = elem_bytes(p);
    const bool inside = R0 + kPackBlock <= rows && C0 + kPackBlock <= cols;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int r = t / 16 + 16 * it, c4 = (t % 16) * 4;
        const double2 *src = (const double2 *)(X + (R0 + r) * ld + C0 + c4);
        double2 x01 = make_double2(0.0, 0.0), x23 = x01;
        if (inside) {
            x01 = src[0];
            x23 = src[1];
        } else if (R0 + r < rows) {
            // pairs are read whole where the row's allocation (ld entries, ld even) holds them
            const int64_t c = C0 + c4;
            if (c < cols) { x01 = src[0]; if (c + 1 >= cols) x01.y = 0.0; }
            if (c + 2 < cols) { x23 = src[1]; if (c + 3 >= cols) x23.y = 0.0; }
        }
        uint64_t b[4] = {stored_bits(x01.x, p, e), stored_bits(x01.y, p, e),
                         stored_bits(x23.x, p, e), stored_bits(x23.y, p, e)};
        if (!TRANSPOSE) {
            store4(base + ((int64_t)(r_in + r) * nb + c_in + c4) * es, p, b);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) turn[c4 + j][r] = b[j];
        }
    }
    if (TRANSPOSE) {
        __syncthreads();
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int c = t / 16 + 16 * it, r4 = (t % 16) * 4;
            uint64_t b[4] = {turn[c][r4], turn[c][r4 + 1], turn[c][r4 + 2], turn[c][r4 + 3]};
            store4(base + ((int64_t)(c_in + c) * nb + r_in + r4) * es, p, b);
        }
    }
}

// rows x cols, rows_t x cols_t: the buffer as it lies in memory.  turn: the rows of a packed tile
// are the buffer's columns; swap: tile (I, J) of the buffer is tile (J, I) of the matrix.
hipError_t launch_pack(const double *X, int64_t ld, int64_t rows, int64_t cols, int rows_t, int cols_t, int nb, bool turn,
                       bool swap, PackedView v, hipStream_t s)
{
    dim3 grid((unsigned)((int64_t)cols_t * nb / kPackBlock), (unsigned)((int64_t)rows_t * nb / kPackBlock));
    if (turn) pack_kernel<true><<<grid, 256, 0, s>>>(X, ld, rows, cols, nb, rows_t, cols_t, swap, v);
    else pack_kernel<false><<<grid, 256, 0, s>>>(X, ld, rows, cols, nb, rows_t, cols_t, swap, v);
    return hipGetLastError();
}

// Block-scaled tiles (MXFP8, MXFP4, MXFP6: the formats of the OCP microscaling specification): per block
// of 32 consecutive reduction indices of one packed row (a row of an A tile, a column of a B
// tile) a scale 2^s, s = floor(log2 max|x|) - 8 (e4m3 elements) or - 2 (e2m1, e2m3) within [-127, 127]
// (0 for a zero block or a non-finite maximum); elements x * 2^-s rounded once, saturating; the
// scale bytes (s + 127) follow the tile's element bytes, nb / 32 per packed row.  Entries outside
// the rows x cols matrix count as zeros.
// Scale exponent of a block from its largest magnitude (narrow: e2m1 or e2m3 elements, whose
// largest binade is 4 .. 8; else e4m3).
__device__ inline int mx_block_exponent(double m, bool narrow)
{
    const uint64_t bits = (uint64_t)__double_as_longlong(m);
    const int field = (int)(bits >> 52);
    const uint64_t man = bits & 0xfffffffffffffull;
    if (field == 0x7ff || bits == 0) return 0;
    const int lg = field ? field - 1023 : 63 - __builtin_clzll(man) - 1074;
    const int s = lg - (narrow ? 2 : 8);                            // exponent of the element format's largest binade
    return s < -127 ? -127 : s > 127 ? 127 : s;
}

// B tiles (blocks run down the matrix columns): one thread per block, neighbouring threads on
// neighbouring columns, so that every load of a wave is 512 contiguous bytes.
__global__ __launch_bounds__(256) void pack_mx_kernel(const double *__restrict__ X, int64_t sr, int64_t sc, int64_t rows, int64_t cols,
                                                      int cols_t, int nb, bool is_b, PackedView v)
{
    const unsigned per_tile = (unsigned)(nb * nb / 32 / 256);    // workgroups per tile; the grid is one-dimensional
    const int tile = (int)(blockIdx.x / per_tile);
    const int p = v.prec[tile];
    if (!is_block_scaled(p)) return;
    const bool fp4 = p == GEMM_MP_MXFP4, fp6 = p == GEMM_MP_MXFP6;
    const int I = tile / cols_t, J = tile % cols_t;
    const int per_row = nb / 32;
    const int idx = (int)(blockIdx.x % per_tile) * 256 + threadIdx.x;   // (block, packed row): nb * nb / 32 of them, a multiple of 256
    const int u = is_b ? idx % nb : idx / per_row, kb = is_b ? idx / nb : idx % per_row;
    double x[32];
    double m = 0.0;
#pragma unroll
    for (int k = 0; k < 32; ++k) {
        const int64_t r = (int64_t)I * nb + (is_b ? 32 * kb + k : u), c = (int64_t)J * nb + (is_b ? u : 32 * kb + k);
        x[k] = (r < rows && c < cols) ? X[r * sr + c * sc] : 0.0;
        const double a = __builtin_fabs(x[k]);
        if (a > m) m = a;                                        // a NaN never enters m
    }
    const int s = mx_block_exponent(m, fp4 || fp6);
    char *base = v.storage + v.offset[tile];
    if (fp6) {                                                   // 32 six-bit codes in 24 bytes, code k at bits 6k .. 6k+5
        uint64_t w[3] = {0, 0, 0};
#pragma unroll
        for (int k = 0; k < 32; ++k) {
            const uint64_t code = to_fp6_bits(x[k], s);
            w[(6 * k) / 64] |= code << ((6 * k) % 64);
            if ((6 * k) % 64 > 58) w[(6 * k) / 64 + 1] |= code >> (64 - (6 * k) % 64);
        }
        uint2 *dst = (uint2 *)(base + fp6_group_offset(nb, u, 32 * kb));
#pragma unroll
        for (int j = 0; j < 3; ++j) dst[j] = make_uint2((uint32_t)w[j], (uint32_t)(w[j] >> 32));
        ((uint8_t *)base)[(int64_t)nb * nb / 4 * 3 + (int64_t)u * per_row + kb] = (uint8_t)(s + 127);
        return;
    }
    if (fp4) {                                                   // two elements a byte, the lower index in the low four bits
        uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
        for (int k = 0; k < 32; ++k) w[k / 8] |= to_fp4_bits(x[k], s) << (4 * (k % 8));
        *(uint4 *)(base + ((int64_t)u * nb + 32 * kb) / 2) = make_uint4(w[0], w[1], w[2], w[3]);
        ((uint8_t *)base)[(int64_t)nb * nb / 2 + (int64_t)u * per_row + kb] = (uint8_t)(s + 127);
        return;
    }
    uint32_t w[8];
#pragma unroll
    for (int k = 0; k < 32; k += 4)
        w[k / 4] = to_fp8_bits(x[k], s) | (to_fp8_bits(x[k + 1], s) << 8) | (to_fp8_bits(x[k + 2], s) << 16) | (to_fp8_bits(x[k + 3], s) << 24);
    uint4 *dst = (uint4 *)(base + (int64_t)u * nb + 32 * kb);
    dst[0] = make_uint4(w[0], w[1], w[2], w[3]);
    dst[1] = make_uint4(w[4], w[5], w[6], w[7]);
    ((uint8_t *)base)[(int64_t)nb * nb + (int64_t)u * per_row + kb] = (uint8_t)(s + 127);
}

// A tiles (blocks run along the matrix rows): eight neighbouring lanes share a block, four
// consecutive entries each, so that a wave reads 2 KB of a row at a time; the block maximum is
// formed with three lane exchanges.
__global__ __launch_bounds__(256) void pack_mx_rows_kernel(const double *__restrict__ X, int64_t sr, int64_t sc, int64_t rows, int64_t cols,
                                                           int cols_t, int nb, PackedView v)
{
    const unsigned per_tile = (unsigned)(nb * nb / 4 / 256);     // workgroups per tile; the grid is one-dimensional
    const int tile = (int)(blockIdx.x / per_tile);
    const int p = v.prec[tile];
    if (!is_block_scaled(p)) return;
    const bool fp4 = p == GEMM_MP_MXFP4, fp6 = p == GEMM_MP_MXFP6;
    const int I = tile / cols_t, J = tile % cols_t;
    const int per_row = nb / 32;
    const int gidx = (int)(blockIdx.x % per_tile) * 256 + threadIdx.x;   // (block, quarter of eight): nb * nb / 4 of them
    const int blk = gidx >> 3, sub = gidx & 7;
    const int u = blk / per_row, kb = blk % per_row;
    const int64_t r = (int64_t)I * nb + u, c0 = (int64_t)J * nb + 32 * kb + 4 * sub;
    double x[4];
    double m = 0.0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        x[k] = (r < rows && c0 + k < cols) ? X[r * sr + (c0 + k) * sc] : 0.0;
        const double a = __builtin_fabs(x[k]);
        if (a > m) m = a;
    }
#pragma unroll
    for (int d = 1; d < 8; d <<= 1) {
        const double o = __shfl_xor(m, d);
        if (o > m) m = o;
    }
    const int s = mx_block_exponent(m, fp4 || fp6);
    char *base = v.storage + v.offset[tile];
    if (fp6) {                                                   // four codes = three bytes
        const uint32_t w = to_fp6_bits(x[0], s) | (to_fp6_bits(x[1], s) << 6) | (to_fp6_bits(x[2], s) << 12) | (to_fp6_bits(x[3], s) << 18);
        uint8_t *d = (uint8_t *)base + fp6_group_offset(nb, u, 32 * kb + 4 * sub);
        d[0] = (uint8_t)w; d[1] = (uint8_t)(w >> 8); d[2] = (uint8_t)(w >> 16);
        if (sub == 0) ((uint8_t *)base)[(int64_t)nb * nb / 4 * 3 + (int64_t)u * per_row + kb] = (uint8_t)(s + 127);
        return;
    }
    if (fp4) {
        const uint32_t w = to_fp4_bits(x[0], s) | (to_fp4_bits(x[1], s) << 4) | (to_fp4_bits(x[2], s) << 8) | (to_fp4_bits(x[3], s) << 12);
        *(uint16_t *)(base + ((int64_t)u * nb + 32 * kb) / 2 + 2 * sub) = (uint16_t)w;
        if (sub == 0) ((uint8_t *)base)[(int64_t)nb * nb / 2 + (int64_t)u * per_row + kb] = (uint8_t)(s + 127);
        return;
    }
    const uint32_t w = to_fp8_bits(x[0], s) | (to_fp8_bits(x[1], s) << 8) | (to_fp8_bits(x[2], s) << 16) | (to_fp8_bits(x[3], s) << 24);
    *(uint32_t *)(base + (int64_t)u * nb + 32 * kb + 4 * sub) = w;
    if (sub == 0) ((uint8_t *)base)[(int64_t)nb * nb + (int64_t)u * per_row + kb] = (uint8_t)(s + 127);
}

hipError_t launch_pack_mx(const double *X, int64_t sr, int64_t sc, int64_t rows, int64_t cols, int rows_t, int cols_t, int nb,
                          bool is_b, PackedView v, hipStream_t s)
{
    // the mapping that reads contiguously: by the direction in which the buffer is contiguous along the blocks
    const bool along_contiguous = is_b ? sr == 1 : sc == 1;
    if (along_contiguous && !is_b) {
        const int64_t blocks = (int64_t)nb * nb / 4 / 256 * rows_t * cols_t;
        if (blocks > 0x7fffffff) return hipErrorInvalidValue;
        dim3 grid((unsigned)blocks);
        pack_mx_rows_kernel<<<grid, 256, 0, s>>>(X, sr, sc, rows, cols, cols_t, nb, v);
    } else {
        const int64_t blocks = (int64_t)nb * nb / 32 / 256 * rows_t * cols_t;
        if (blocks > 0x7fffffff) return hipErrorInvalidValue;
        dim3 grid((unsigned)blocks);
        pack_mx_kernel<<<grid, 256, 0, s>>>(X, sr, sc, rows, cols, cols_t, nb, is_b, v);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Unpack: the exact FP64 value of every stored element (stored number times 2^e; for an MXFP8
// tile of size nb, times the scale of its block of 32).
__device__ inline double stored_value(const char *base, int64_t idx, int p, int e, int nb)
{
    switch (p) {
    case GEMM_MP_MXFP8: {
        const int code = ((const uint8_t *)base)[idx];
        const int sc = ((const uint8_t *)base)[(int64_t)nb * nb + (idx >> 5)];
        return ldexp((double)__builtin_amdgcn_cvt_f32_fp8(code, 0), sc - 127);
    }
    case GEMM_MP_MXFP4: {
        const int code = (((const uint8_t *)base)[idx >> 1] >> (4 * (int)(idx & 1))) & 15;
        const int sc = ((const uint8_t *)base)[(int64_t)nb * nb / 2 + (idx >> 5)];
        const int ef = (code >> 1) & 3, mf = code & 1;
        const double mag = ef ? ldexp(1.0 + 0.5 * mf, ef - 1) : 0.5 * mf;
        return ldexp((code & 8) ? -mag : mag, sc - 127);
    }
    case GEMM_MP_MXFP6: {
        const int64_t at = fp6_group_offset(nb, (int)(idx / nb), (int)(idx % nb) & ~3);   // four codes = three bytes
        const uint32_t w = ((const uint8_t *)base)[at] | ((uint32_t)((const uint8_t *)base)[at + 1] << 8) | ((uint32_t)((const uint8_t *)base)[at + 2] << 16);
        const int sc = ((const uint8_t *)base)[(int64_t)nb * nb / 4 * 3 + (idx >> 5)];
        return ldexp((double)fp6_value((w >> (6 * (int)(idx & 3))) & 63u), sc - 127);
    }
    case GEMM_MP_FP64: return ((const double *)base)[idx];
    case GEMM_MP_FP32: return (double)((const float *)base)[idx];
    case GEMM_MP_FP16: return ldexp((double)(float)((const _Float16 *)base)[idx], e);
    case GEMM_MP_BF16: return (double)__uint_as_float((uint32_t)((const uint16_t *)base)[idx] << 16);
    default: {
        const int code = ((const uint8_t *)base)[idx];
        return ldexp((double)__builtin_amdgcn_cvt_f32_fp8(code, 0), e);
    }
    }
}

// Only the rows x cols entries of the matrix are written.
template <bool TRANSPOSE>
__global__ __launch_bounds__(256) void unpack_kernel(double *__restrict__ X, int64_t ld, int64_t rows, int64_t cols, int nb,
                                                     int rows_t, int cols_t, bool swap, PackedView v)
{
    __shared__ double turn[TRANSPOSE ? kPackBlock : 1][TRANSPOSE ? kPackBlock + 1 : 1];
    const int t = threadIdx.x;
    const int64_t R0 = (int64_t)blockIdx.y * kPackBlock, C0 = (int64_t)blockIdx.x * kPackBlock;
    const int I = (int)(R0 / nb), J = (int)(C0 / nb);
    const int tile = swap ? J * rows_t + I : I * cols_t + J;      // swap: the buffer holds the matrix's transpose
    const int p = v.prec[tile];
    const int e = v.exp[tile];
    const char *base = v.storage + v.offset[tile];
    const int r_in = (int)(R0 % nb), c_in = (int)(C0 % nb);
    if (TRANSPOSE) {
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int c = t / 16 + 16 * it, r4 = (t % 16) * 4;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                turn[c][r4 + j] = stored_value(base, (int64_t)(c_in + c) * nb + r_in + r4 + j, p, e, nb);
        }
        __syncthreads();
    }
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int r = t / 16 + 16 * it, c4 = (t % 16) * 4;
        double x[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            x[j] = TRANSPOSE ? turn[c4 + j][r]
                             : stored_value(base, (int64_t)(r_in + r) * nb + c_in + c4 + j, p, e, nb);
        if (R0 + kPackBlock <= rows && C0 + kPackBlock <= cols) {
            double2 *dst = (double2 *)(X + (R0 + r) * ld + C0 + c4);
            dst[0] = make_double2(x[0], x[1]);
            dst[1] = make_double2(x[2], x[3]);
        } else if (R0 + r < rows) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (C0 + c4 + j < cols) X[(R0 + r) * ld + C0 + c4 + j] = x[j];
        }
    }
}

hipError_t launch_unpack(double *X, int64_t ld, int64_t rows, int64_t cols, int rows_t, int cols_t, int nb, bool turn,
                         bool swap, PackedView v, hipStream_t s)
{
    dim3 grid((unsigned)((int64_t)cols_t * nb / kPackBlock), (unsigned)((int64_t)rows_t * nb / kPackBlock));
    if (turn) unpack_kernel<true><<<grid, 256, 0, s>>>(X, ld, rows, cols, nb, rows_t, cols_t, swap, v);
    else unpack_kernel<false><<<grid, 256, 0, s>>>(X, ld, rows, cols, nb, rows_t, cols_t, swap, v);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// C tiles stored in FP16 / FP8.  Such a tile is accumulated like an FP32 tile, in an FP32
// staging copy behind the packed tiles of C; around the GEMM kernels three streaming passes,
// one workgroup per kLowChunk consecutive elements of one such tile, connect the two forms:
//   expand  (only when beta != 0): staging = stored number * 2^e, exact;
//   maximum: largest magnitude per chunk, then per tile, and from it the tile's new exponent
//            by the same rule as for packed operands;
//   round:   stored number = staging * 2^-e rounded once to nearest even (FP8 saturates).
__global__ __launch_bounds__(256) void low_expand_kernel(const LowTile *__restrict__ low, PackedView v, int nb)
{
    const unsigned parts = (unsigned)(nb * nb / kLowChunk);     // workgroups per tile; the grid is one-dimensional
    const LowTile lt = low[blockIdx.x / parts];
    const int p = v.prec[lt.tile];
    int e = v.exp[lt.tile];
    const char *src = v.storage + v.offset[lt.tile];
    float *dst = (float *)(v.storage + lt.stage);
    const int64_t i0 = (int64_t)(blockIdx.x % parts) * kLowChunk + threadIdx.x * 4;
#pragma unroll
    for (int it = 0; it < kLowChunk / 1024; ++it) {
        const int64_t i = i0 + it * 1024;
        float4 x;
        if (p == GEMM_MP_FP16) {
            const uint2 h = *(const uint2 *)(src + i * 2);
            const _Float16 *hh = (const _Float16 *)&h;
            x = make_float4((float)hh[0], (float)hh[1], (float)hh[2], (float)hh[3]);
        } else if (p == GEMM_MP_BF16) {
            const uint2 h = *(const uint2 *)(src + i * 2);
            x = make_float4(__uint_as_float(h.x << 16), __uint_as_float(h.x & 0xffff0000u),
                            __uint_as_float(h.y << 16), __uint_as_float(h.y & 0xffff0000u));
        } else if (p == GEMM_MP_MXFP6) {                       // four codes = three bytes, in one block of 32
            const uint8_t *b3 = (const uint8_t *)src + fp6_group_offset(nb, (int)(i / nb), (int)(i % nb));
            const uint32_t b = b3[0] | ((uint32_t)b3[1] << 8) | ((uint32_t)b3[2] << 16);
            x = make_float4(fp6_value(b & 63u), fp6_value((b >> 6) & 63u), fp6_value((b >> 12) & 63u), fp6_value((b >> 18) & 63u));
            e = (int)((const uint8_t *)src)[(int64_t)nb * nb / 4 * 3 + (i >> 5)] - 127;
        } else if (p == GEMM_MP_MXFP4) {                       // the four entries share one block of 32
            const uint32_t b = *(const uint16_t *)(src + i / 2);
            float m[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t code = (b >> (4 * j)) & 15u;
                const int ef = (code >> 1) & 3, mf = code & 1;
                const float mag = ef ? ldexpf(1.0f + 0.5f * mf, ef - 1) : 0.5f * mf;
                m[j] = (code & 8u) ? -mag : mag;
            }
            x = make_float4(m[0], m[1], m[2], m[3]);
            e = (int)((const uint8_t *)src)[(int64_t)nb * nb / 2 + (i >> 5)] - 127;
        } else {
            const uint32_t b = *(const uint32_t *)(src + i);
            if (p == GEMM_MP_MXFP8) e = (int)((const uint8_t *)src)[(int64_t)nb * nb + (i >> 5)] - 127;
            x = make_float4(__builtin_amdgcn_cvt_f32_fp8(b, 0), __builtin_amdgcn_cvt_f32_fp8(b, 1),
                            __builtin_amdgcn_cvt_f32_fp8(b, 2), __builtin_amdgcn_cvt_f32_fp8(b, 3));
        }
        x.x = ldexpf(x.x, e); x.y = ldexpf(x.y, e); x.z = ldexpf(x.z, e); x.w = ldexpf(x.w, e);
        *(float4 *)(dst + i) = x;
    }
}

__global__ __launch_bounds__(256) void low_chunk_max_kernel(const LowTile *__restrict__ low, const char *__restrict__ storage,
                                                            int parts, float *__restrict__ part_max)
{
    __shared__ float wm[4];
    const LowTile lt = low[blockIdx.x / (unsigned)parts];
    const float *src = (const float *)(storage + lt.stage);
    const int64_t i0 = (int64_t)(blockIdx.x % (unsigned)parts) * kLowChunk + threadIdx.x * 4;
    float m = 0.0f;
#pragma unroll
    for (int it = 0; it < kLowChunk / 1024; ++it) {
        const float4 x = *(const float4 *)(src + i0 + it * 1024);
        const float a[4] = {__builtin_fabsf(x.x), __builtin_fabsf(x.y), __builtin_fabsf(x.z), __builtin_fabsf(x.w)};
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (a[j] > m) m = a[j];          // a NaN never enters m
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const float o = __shfl_xor(m, d);
        if (o > m) m = o;
    }
    if ((threadIdx.x & 63) == 0) wm[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int k = 1; k < 4; ++k)
            if (wm[k] > m) m = wm[k];
        part_max[blockIdx.x] = m;                      // = tile * parts + chunk
    }
}

__global__ __launch_bounds__(256) void low_exponent_kernel(const LowTile *__restrict__ low, const uint8_t *__restrict__ prec,
                                                           int parts, const float *__restrict__ part_max,
                                                           int32_t *__restrict__ exps)
{
    __shared__ float wm[4];
    const LowTile lt = low[blockIdx.x];
    float m = 0.0f;
    for (int k = threadIdx.x; k < parts; k += 256) {
        const float x = part_max[(int64_t)blockIdx.x * parts + k];
        if (x > m) m = x;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const float o = __shfl_xor(m, d);
        if (o > m) m = o;
    }
    if ((threadIdx.x & 63) == 0) wm[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int k = 1; k < 4; ++k)
            if (wm[k] > m) m = wm[k];
        const uint32_t bits = __float_as_uint(m);
        const int field = (int)(bits >> 23);
        const uint32_t man = bits & 0x7fffffu;
        int e = 0;
        if (field != 0xff && bits != 0 && prec[lt.tile] != GEMM_MP_BF16 && !is_block_scaled(prec[lt.tile])) {
            // (BF16 tiles carry no scale, block-scaled tiles none for the whole tile)
            const int lg = field ? field - 127 : 31 - __builtin_clz(man) - 149;
            e = lg - (prec[lt.tile] == GEMM_MP_FP16 ? 14 : 7);
        }
        exps[lt.tile] = e;
    }
}

__global__ __launch_bounds__(256) void low_round_kernel(const LowTile *__restrict__ low, PackedView v, int nb)
{
    const unsigned parts = (unsigned)(nb * nb / kLowChunk);     // workgroups per tile; the grid is one-dimensional
    const LowTile lt = low[blockIdx.x / parts];
    const int p = v.prec[lt.tile];
    const int e = v.exp[lt.tile];
    char *dst = v.storage + v.offset[lt.tile];
    const float *src = (const float *)(v.storage + lt.stage);
    const int es = elem_bytes(p);
    const int64_t i0 = (int64_t)(blockIdx.x % parts) * kLowChunk + threadIdx.x * 4;
#pragma unroll
    for (int it = 0; it < kLowChunk / 1024; ++it) {
        const int64_t i = i0 + it * 1024;
        const float4 x = *(const float4 *)(src + i);
        if (is_block_scaled(p)) {                            // uniform over the workgroup
            // eight neighbouring lanes hold one block of 32 along a row of the tile
            const bool fp4 = p == GEMM_MP_MXFP4, fp6 = p == GEMM_MP_MXFP6;
            float m = __builtin_fabsf(x.x);
            const float a[3] = {__builtin_fabsf(x.y), __builtin_fabsf(x.z), __builtin_fabsf(x.w)};
            if (!(m == m)) m = 0.0f;                         // a NaN never enters m
#pragma unroll
            for (int j = 0; j < 3; ++j)
                if (a[j] > m) m = a[j];
#pragma unroll
            for (int d = 1; d < 8; d <<= 1) {
                const float o = __shfl_xor(m, d);
                if (o > m) m = o;
            }
            const int s = mx_block_exponent((double)m, fp4 || fp6);
            if (fp6) {
                const uint32_t w = to_fp6_bits((double)x.x, s) | (to_fp6_bits((double)x.y, s) << 6) |
                                   (to_fp6_bits((double)x.z, s) << 12) | (to_fp6_bits((double)x.w, s) << 18);
                uint8_t *d = (uint8_t *)dst + fp6_group_offset(nb, (int)(i / nb), (int)(i % nb));
                d[0] = (uint8_t)w; d[1] = (uint8_t)(w >> 8); d[2] = (uint8_t)(w >> 16);
                if ((threadIdx.x & 7) == 0) ((uint8_t *)dst)[(int64_t)nb * nb / 4 * 3 + (i >> 5)] = (uint8_t)(s + 127);
            } else if (fp4) {
                const uint32_t w = to_fp4_bits((double)x.x, s) | (to_fp4_bits((double)x.y, s) << 4) |
                                   (to_fp4_bits((double)x.z, s) << 8) | (to_fp4_bits((double)x.w, s) << 12);
                *(uint16_t *)(dst + i / 2) = (uint16_t)w;
                if ((threadIdx.x & 7) == 0) ((uint8_t *)dst)[(int64_t)nb * nb / 2 + (i >> 5)] = (uint8_t)(s + 127);
            } else {
                const uint32_t w = to_fp8_bits((double)x.x, s) | (to_fp8_bits((double)x.y, s) << 8) |
                                   (to_fp8_bits((double)x.z, s) << 16) | (to_fp8_bits((double)x.w, s) << 24);
                *(uint32_t *)(dst + i) = w;
                if ((threadIdx.x & 7) == 0) ((uint8_t *)dst)[(int64_t)nb * nb + (i >> 5)] = (uint8_t)(s + 127);
            }
            continue;
        }
        const uint64_t b[4] = {stored_bits((double)x.x, p, e), stored_bits((double)x.y, p, e),
                               stored_bits((double)x.z, p, e), stored_bits((double)x.w, p, e)};
        store4(dst + i * es, p, b);
    }
}

hipError_t launch_low_expand(const LowTile *low_dev, int n_low, int nb, PackedView c, hipStream_t s)
{
    if (n_low == 0) return hipSuccess;
    const int64_t blocks = (int64_t)nb * nb / kLowChunk * n_low;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    dim3 grid((unsigned)blocks);
    low_expand_kernel<<<grid, 256, 0, s>>>(low_dev, c, nb);
    return hipGetLastError();
}

hipError_t launch_low_store(const LowTile *low_dev, int n_low, int nb, PackedView c, int32_t *exps, float *part_max,
                            hipStream_t s)
{
    if (n_low == 0) return hipSuccess;
    const int parts = (int)((int64_t)nb * nb / kLowChunk);
    if ((int64_t)parts * n_low > 0x7fffffff) return hipErrorInvalidValue;
    dim3 grid((unsigned)((int64_t)parts * n_low));
    low_chunk_max_kernel<<<grid, 256, 0, s>>>(low_dev, c.storage, parts, part_max);
    low_exponent_kernel<<<n_low, 256, 0, s>>>(low_dev, c.prec, parts, part_max, exps);
    low_round_kernel<<<grid, 256, 0, s>>>(low_dev, c, nb);
    return hipGetLastError();
}

}  // namespace gmp
