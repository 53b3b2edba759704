/*
 * gemm_mp.h - C ABI of the tile-centric mixed-precision GEMM for one MI355X (gfx950).
 *
 *     C <- alpha * A * B + beta * C          (paper Section 4, Algorithm 1)
 *
 * A (M x K), B (K x N) and C (M x N) are cut into square tiles of one size
 * tile_nb.  Every tile is stored in its own precision, given per matrix by a
 * precision map (one unsigned 16-bit code per tile, row-major over tiles;
 * paper Section 5.2).  A tile product A(I,L)*B(L,J) is computed on the matrix
 * cores at the precision the policy assigns to it, operands being converted
 * from their stored precision on the fly by the consumer ("receiver-side
 * conversion", Section 4), and is accumulated into C(I,J) in that tile's
 * precision.  Each C tile region is owned by exactly one workgroup: there are
 * no atomics on C and results are reproducible run to run.
 *
 * Conventions
 *   - Dense matrices handed to / returned by the library are row-major FP64 in
 *     DEVICE memory, leading dimension `ld` in elements.
 *   - Precision maps and everything returned through pointers marked "host"
 *     live in HOST memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls marked [async] only enqueue work on it (kernels and small
 *     host-to-device copies from pinned memory that the library owns); calls
 *     marked [sync] wait for it before they return.  The [async] calls on one
 *     context must be issued on one stream, or on streams the caller has
 *     ordered: each reads what the one before it queued.  The first [async]
 *     call that meets a new shape allocates the library's tables (which waits
 *     for the device); afterwards a context that sees maps of the same shapes
 *     again allocates nothing and waits for nothing in those calls.
 *   - The library never allocates or frees operand memory.  The caller asks
 *     gemm_mp_storage_bytes() and binds a device buffer of at least that size
 *     per matrix; the buffer must stay valid until the context is destroyed or
 *     rebound.  The library owns only small per-tile tables.
 *   - Every entry point returns a status code (0 = success).  Nothing throws or
 *     aborts.  Output arguments are written only on success.
 *   - A context must not be used from two threads at once.
 *
 * Packed layout of a matrix (what the bound buffer holds): tile (I,J) starts at
 * a 256-byte aligned offset, tiles in row-major order; inside a tile of A or C
 * element (r,c) sits at index r*tile_nb + c; inside a tile of B at index
 * c*tile_nb + r (so the reduction index is contiguous for both operands).
 * Element types: FP64 / FP32 IEEE; FP16 IEEE binary16; FP8 OCP e4m3 ("fn": no
 * infinities, max finite 448).  FP16 / FP8 tiles hold x * 2^-e with one
 * power-of-two exponent e per tile chosen so that the largest magnitude falls
 * in [2^14,2^15) resp. [2^7,2^8); e = 0 for an all-zero tile.  BF16 tiles (8
 * exponent bits as FP32, 7 fraction bits, overflow to infinity) have FP32's
 * range and carry no scale (e = 0).  MXFP8 tiles (code 5) are the block-scaled
 * format of the OCP microscaling specification: e4m3 elements, tile_nb^2 bytes laid out like an
 * FP8 tile, followed by one scale byte (E8M0: 2^(code-127)) per 32 consecutive reduction
 * indices, row by row, tile_nb^2/32 bytes; scale = 2^(floor(log2 max|x|) - 8) of its block,
 * elements rounded once and saturating; no tile scale.  Where every product of a C tile is
 * MXFP8 x MXFP8 (C tile not FP64, tile_nb a multiple of 256) the tile runs on the block-scaled
 * matrix instruction; under any other product an MXFP8 tile is widened by the receiving
 * workgroup (element times block scale): see gemm_mp_run.  MXFP4 tiles (code 6)
 * are the same with e2m1 elements (magnitudes 0, 0.5, 1, 1.5, 2, 3, 4, 6; scale
 * 2^(floor(log2 max|x|) - 2)): tile_nb^2/2 element bytes, two elements per byte with the lower
 * reduction index in the low four bits, then the tile_nb^2/32 scale bytes; block-scaled
 * instruction where every product of a C tile is MXFP4 x MXFP4 and tile_nb is a multiple of 512.
 * MXFP6 tiles (code 7) are the same with e2m3 elements (six bits: sign, two exponent bits with
 * bias 1, three fraction bits; the magnitudes are the multiples of 1/8 below 2, of 1/4 below 4 and
 * of 1/2 up to 7.5; scale 2^(floor(log2 max|x|) - 2)): 3*tile_nb^2/4 element bytes, a block of 32
 * elements being 24 bytes with element k of the block in bits 6k .. 6k+5 (least significant bit
 * first, as the matrix instruction reads them), then the tile_nb^2/32 scale bytes, row by row.  The
 * element bytes are laid out for the kernel that multiplies them: panel by panel of 128 reduction
 * indices; inside a panel row after row (96 bytes each); inside a row of a panel, block b of the
 * panel's four at block position (b + row/8) mod 4.  Block-scaled instruction
 * where every product of a C tile is MXFP6 x MXFP6 and tile_nb is a multiple of 256.
 *
 * C tiles stored in FP16 / FP8 (formats beyond FP64 / FP32 are what the paper's
 * Section 6 leaves open): such a tile is a storage format only.  Its products
 * get the precisions an FP32 tile's would and it is accumulated in FP32; when
 * the tile is finished its largest magnitude fixes a new exponent e by the rule
 * above and every entry is rounded once more, from FP32, to nearest even.  With
 * beta != 0 the old tile enters as stored number * 2^e.  BF16 C tiles are rounded
 * without a scale; MXFP8 / MXFP4 / MXFP6 C tiles are quantised block by block, the blocks
 * of 32 running along the rows of the tile as in a tile of A.  The FP32 form lives in
 * a staging copy per such tile that follows the packed tiles in C's buffer
 * (gemm_mp_storage_bytes counts it), so the library still allocates no operand
 * memory; only gemm_mp_run touches the staging area.
 */
#ifndef GEMM_MP_H
#define GEMM_MP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gemm_mp_ctx gemm_mp_ctx; /* opaque; created and destroyed by the library */
typedef void *gemm_mp_stream;           /* a hipStream_t */

/* Precision codes of a map entry: 0 and 1 as in the paper (Section 5.2); 2, 3, 4 extend them.
 * The code is a name, not a rank: by unit roundoff (2^-53, 2^-24, 2^-11, 2^-8, 2^-4) the formats
 * order FP64, FP32, FP16, BF16, FP8. */
enum { GEMM_MP_FP64 = 0, GEMM_MP_FP32 = 1, GEMM_MP_FP16 = 2, GEMM_MP_FP8_E4M3 = 3, GEMM_MP_BF16 = 4,
       GEMM_MP_MXFP8 = 5, GEMM_MP_MXFP4 = 6, GEMM_MP_MXFP6 = 7 };

enum {
    GEMM_MP_OK = 0,
    GEMM_MP_EINVAL = -1,       /* bad argument: null pointer, size, letter, map code, alignment */
    GEMM_MP_ESTATE = -2,       /* call order: a map, a buffer or packed data is missing */
    GEMM_MP_ENOMEM = -3,       /* a table could not be allocated */
    GEMM_MP_EUNSUPPORTED = -4, /* valid request this build does not implement */
    GEMM_MP_EHIP = -5,         /* the HIP runtime reported an error */
    GEMM_MP_ETOOBIG = -6       /* gemm_mp_run_static: more tile products than its static scratch holds */
};

/* How the precision q of the product A(I,L)*B(L,J) that updates C(I,J) is chosen.
 *   OPERAND (default): the better of the two operands' stored precisions, but never above
 *       the type the C tile is accumulated in: q = min(cap(pC), max(pA,pB)), cap(FP64)=FP64,
 *       else FP32.  With BF16 "the better" is the smallest format that holds both operands'
 *       numbers exactly, FP64 > FP32 > {FP16, BF16} > FP8: FP32 for an FP16 with a BF16 tile,
 *       BF16 for a BF16 with a BF16 or an FP8 tile.  A BF16 product multiplies on the BF16
 *       matrix instruction with FP32 accumulation, like an FP16 one.
 *   C_TILE: the paper's literal statement (Section 5.2: the result precision follows the C
 *       tile and operands are converted when their maps differ): q = cap(pC), which is pC
 *       itself on the paper's FP64 / FP32 maps.
 * The two agree on FP64/FP32 maps except for (pA,pB,pC) = (FP32,FP32,FP64). */
enum { GEMM_MP_POLICY_OPERAND = 0, GEMM_MP_POLICY_C_TILE = 1 };

typedef struct gemm_mp_stats {
    int64_t products[4];     /* tile products per product precision (index = precision code) */
    double flops[4];         /* 2*nb^3 * products[q] */
    int64_t tiles[3][4];     /* stored tiles per matrix (0=A,1=B,2=C) and precision */
    uint64_t packed_bytes[3];/* size of the packed buffer per matrix */
    int64_t work_items;      /* owner workgroups launched by gemm_mp_run */
    int64_t converted_tiles; /* tile copies the sender-side workspace holds (0: receiver-side) */
    uint64_t converted_bytes;/* their total size */
    int64_t products_bf16;   /* the same counts for precision code 4, kept apart so that the */
    double flops_bf16;       /* arrays above stay indexed by the codes 0..3 */
    int64_t tiles_bf16[3];
    int64_t products_mxfp8;  /* the same for precision code 5 */
    double flops_mxfp8;
    int64_t tiles_mxfp8[3];
    int64_t products_mxfp4;  /* the same for precision code 6 */
    double flops_mxfp4;
    int64_t tiles_mxfp4[3];
    int64_t launch_items[8]; /* owner workgroups per kernel launch of gemm_mp_run: [0] 128 x 128 regions of
                              * FP64 C tiles, [1] of C tiles accumulated in FP32, [2] / [3] / [4] 256 x 256
                              * regions of tiles made of FP8 / MXFP8 / MXFP4 products only, [5] / [6] of FP16 /
                              * BF16 products only, [7] of MXFP6 products only */
    int32_t owner_instance[2]; /* which instance of the 128 x 128 kernel serves [0] and [1]: 0 plain, 1 the one
                              * whose DMA ring also takes FP16 products with an FP8 operand, 2 the one for BF16 and
                              * block-scaled operands, 3 ([0] only) the one for FP64 C tiles without an FP64 product */
    int64_t products_mxfp6;  /* as products_mxfp4, for precision code 7 */
    double flops_mxfp6;
    int64_t tiles_mxfp6[3];
} gemm_mp_stats;

/* Create a context for C(MxN) = A(MxK) * B(KxN) with square tiles of tile_nb (Section 4:
 * tiles of one fixed size).  EINVAL unless all sizes are positive and tile_nb is a multiple of
 * 128 (the owner workgroup's footprint).  M, N, K need not be multiples of tile_nb: a matrix
 * has ceil(rows / tile_nb) x ceil(cols / tile_nb) tiles, and a tile that sticks out over the
 * edge is that tile of the matrix padded with zeros (the paper's experiments use multiples
 * only; zeros add nothing to a product, a norm or a maximum).  Dense matrices are row-major with
 * a leading dimension ld >= cols that is even, 16-byte aligned, rows * ld entries allocated.
 * Host only. */
int gemm_mp_create(gemm_mp_ctx **out, int64_t M, int64_t N, int64_t K, int32_t tile_nb);

/* Release the context and its tables (not the bound buffers). */
int gemm_mp_destroy(gemm_mp_ctx *ctx);

/* Choose the product-precision policy (see above).  Host only. */
int gemm_mp_set_policy(gemm_mp_ctx *ctx, int policy);

/* Transposed operands: declare that the dense buffers of matrix `which` ('A' or 'B'; EINVAL for
 * 'C') hold its transpose, i.e. the K x M array of A^T or the N x K array of B^T, row-major
 * (the paper's routine and experiments are C = A*B with untransposed operands, Section 4;
 * BLAS callers have op(A), op(B)).  Maps, tile indices and the packed layout stay those of the
 * matrix itself, and the tile scan keeps its order of operations (defined on the matrix, not on
 * the buffer); only the addressing of gemm_mp_tile_scan, gemm_mp_compute_precision_map,
 * gemm_mp_pack_tiles and gemm_mp_unpack_tiles changes, whose ld must then be >= the matrix's
 * row count.  Takes effect from the next of those calls.  Host only. */
int gemm_mp_set_transposed(gemm_mp_ctx *ctx, char which, int transposed);

/* Give the precision map of matrix `which` ('A', 'B' or 'C'): rows x cols codes, row-major,
 * host memory, copied (Section 5.2).  rows/cols must equal the matrix's tile counts (EINVAL),
 * codes must be 0..6 (EINVAL).  Any earlier binding and packed
 * data of that matrix are forgotten.  Host only. */
int gemm_mp_set_precision_map(gemm_mp_ctx *ctx, char which, const uint16_t *map_host,
                              int32_t rows, int32_t cols);

/* Tile scan [sync]: per tile of the dense device matrix, the sum of squares and the largest
 * magnitude, written to host arrays of rows x cols doubles (either may be NULL).  The sum of
 * squares of a tile is defined in one order: per tile column a running fused multiply-add
 * down the rows, then the column sums added pairwise, neighbours first, level by level.
 * (The paper draws its maps at random, Section 5.2; this scan feeds the norm rule below.) */
int gemm_mp_tile_scan(gemm_mp_ctx *ctx, char which, const double *dense_dev, int64_t ld,
                      gemm_mp_stream stream, double *sumsq_host, double *maxabs_host);

/* Norm-based precision map [sync]: scan the dense device matrix and store tile T at the lowest
 * precision p allowed by `allowed_mask` (bit p = code p) that satisfies
 *     |T|_F * sqrt(#tiles) / |X|_F <= threshold / u_p   (u = 2^-53, 2^-24, 2^-11, 2^-4, 2^-8
 * for codes 0..4; "lowest" and "highest" go by u),
 * else at the highest allowed one; evaluated on squares in FP64 as
 *     (S_T * #tiles) * (u_p*u_p) <= (threshold*threshold) * S,  S = sum of S_T in tile order.
 * This is the Frobenius-norm tile criterion of the tile-adaptive work the paper builds on
 * (cited in its Sections 1-2); the paper itself leaves selection strategies to future work
 * (Section 6).  The map becomes the matrix's map as by gemm_mp_set_precision_map and is also
 * copied to map_out_host if that is not NULL.  The scale exponents of FP16/FP8 tiles are taken
 * from this scan, so gemm_mp_pack_tiles must then be given the same matrix values. */
int gemm_mp_compute_precision_map(gemm_mp_ctx *ctx, char which, const double *dense_dev,
                                  int64_t ld, double threshold, uint32_t allowed_mask,
                                  gemm_mp_stream stream, uint16_t *map_out_host);

/* Bytes the packed form of matrix `which` needs (for C: plus 4 * tile_nb^2 bytes of staging per
 * FP16 / FP8 tile); ESTATE before its map is set.  Host only. */
int gemm_mp_storage_bytes(gemm_mp_ctx *ctx, char which, size_t *bytes);

/* Bind the caller's device buffer (256-byte aligned, at least storage_bytes) that holds, or
 * will hold, the packed tiles of `which`.  The caller keeps ownership.  Host only. */
int gemm_mp_bind_storage(gemm_mp_ctx *ctx, char which, void *dev_ptr, size_t bytes);

/* Pack [async]: round every element of the dense device matrix once, to nearest even, into
 * its tile's precision (FP16/FP8 after the tile's power-of-two scaling; FP8 saturates) and
 * write it in the packed layout (Section 5.2: values are initialised in the precision their
 * map gives).  ESTATE unless map and buffer are set.  For 'C' this defines the C that beta
 * multiplies; with beta == 0 packing C may be skipped. */
int gemm_mp_pack_tiles(gemm_mp_ctx *ctx, char which, const double *dense_dev, int64_t ld,
                       gemm_mp_stream stream);

/* Prepare [async] (optional): everything gemm_mp_run needs besides the packed data, for the
 * current maps and policy: the schedule (which owner workgroup computes which region of which C
 * tile, the precision of every tile product: the precision-bucketed task lists that stand in for
 * the paper's runtime scheduling, Section 3) is built on the host and its tables are queued for
 * copying on `stream`, and the library's device tables get their size.  gemm_mp_run does the same
 * by itself when it finds it undone; calling this first, outside the timed or latency-critical
 * part, leaves gemm_mp_run with nothing but kernel launches.  ESTATE until all three maps are set. */
int gemm_mp_prepare(gemm_mp_ctx *ctx, gemm_mp_stream stream);

/* Run [async]: C <- alpha*A*B + beta*C on the packed tiles (Algorithm 1; beta is applied once
 * per C tile, as in the definition in Section 4).  For each C tile the reduction tiles L are
 * taken in ascending order; a product whose precision equals the C tile's accumulate type
 * (FP64 for FP64 tiles, FP32 otherwise) continues the running sum inside the matrix
 * instruction, any other product is formed in an FP32 accumulator and added once.  FP16/FP8
 * products use FP32-accumulating matrix instructions on the scaled operands; 2^(eA+eB) is
 * applied to the finished tile product.  alpha, beta are rounded to the accumulate type.
 * beta == 0: C is not read.  alpha == 0: no product is formed.
 * The run is one small table kernel and up to five GEMM launches (by kind of C tile); the
 * launches touch disjoint C tiles and run side by side on streams of the library's own, forked
 * off `stream` and joined to it again inside the call, so the caller sees one stream.  With the
 * environment variable GEMM_MP_SERIAL_LAUNCHES=1 at gemm_mp_create they stay on `stream`, one
 * after the other; C is the same either way.
 * ESTATE unless A and B are packed, C's map and buffer are set, and (beta != 0) C is packed.
 * BF16 / MXFP8 / MXFP4 tiles under an FP32 or FP64 product are widened on the receiving side like
 * the paper's formats (a BF16 number is the upper half of an FP32 word; a block-scaled element
 * times its block's scale is exact in FP32).  A C tile whose products are all MXFP8 x MXFP8 or all
 * MXFP4 x MXFP4 (not an FP64 tile, tile_nb a multiple of 256 resp. 512) runs on the block-scaled
 * matrix instruction; elsewhere a product of two block-scaled tiles is computed as exact FP32
 * products with FP32 accumulation, which is what it is. */
int gemm_mp_run(gemm_mp_ctx *ctx, double alpha, double beta, gemm_mp_stream stream);

/* Run without allocating [async].  For callers that cannot allocate device memory at the point
 * of the call: code under HIP graph capture, tight serving loops, harnesses that forbid it.  The
 * same computation as gemm_mp_run with the same kernels and bit for bit the same C; the one piece
 * of scratch memory the run needs (the product table: one 32-byte record per tile product A(I,L)*
 * B(L,J), filled by a small kernel at the start of the call) lives in a static device array of
 * (GEMM_MP_STATIC_MAX_PRODUCTS + 2) * 32 bytes (2 MiB) that every GPU the library runs on holds
 * until the process ends.  The call itself allocates nothing, frees nothing, copies nothing from
 * the host and waits for nothing: it launches kernels on `stream`.
 *   - ETOOBIG if the problem has more than GEMM_MP_STATIC_MAX_PRODUCTS tile products
 *     (MT * NT * KT), whatever else its state.
 *   - ESTATE unless gemm_mp_prepare has been called (on a stream ordered before `stream`) since the
 *     last change of a map or of the policy, besides what gemm_mp_run asks for.
 *   - Every call on one GPU uses that GPU's one array, from whatever context or thread: calls
 *     whose execution may overlap on a GPU (different streams) race on it; put them on one stream
 *     or order them.  gemm_mp_run has its own table and may overlap with it.  Nothing in the array
 *     has to start at zero: each call writes every record it reads. */
#define GEMM_MP_STATIC_MAX_PRODUCTS 65536
int gemm_mp_run_static(gemm_mp_ctx *ctx, double alpha, double beta, gemm_mp_stream stream);

/* Sender-side conversion (optional).  The paper converts at the receiver: a tile travels in its
 * stored precision and every task that needs another precision converts it again (Section 4,
 * which leaves other conversion strategies to future work, as does Section 6).  These calls
 * add the opposite strategy on one GPU: every A or B tile is converted once per distinct
 * product precision that differs from its stored one, into a caller-owned workspace, and
 * gemm_mp_run then reads the converted copies, so no task converts anything.  The converted
 * values are exactly the ones the receiver-side path produces (exact up-casts with the tile's
 * 2^e applied for FP64/FP32 targets, FP8 -> FP16 keeping the tile's exponent, and the one
 * rounding FP64 -> FP32), so C is the same; what changes is memory (the workspace), one
 * HBM-bound conversion pass, and which chunk loops the products run through.
 *
 * conversion_bytes: size of that workspace for the current maps and policy (0 if no task needs
 * a conversion).  ESTATE until all three maps are set.  Host only.
 * convert_tiles [async]: fill the workspace (256-byte aligned device memory of at least
 * conversion_bytes, owned by the caller, who keeps it alive while it is in use) from the packed
 * A and B.  ESTATE unless A and B are packed.  Afterwards gemm_mp_run uses the copies until a
 * map, the policy or the packed A or B changes, or clear_conversion is called; then it is
 * back to receiver-side conversion without further notice. */
int gemm_mp_conversion_bytes(gemm_mp_ctx *ctx, size_t *bytes);
int gemm_mp_convert_tiles(gemm_mp_ctx *ctx, void *workspace_dev, size_t bytes, gemm_mp_stream stream);
int gemm_mp_clear_conversion(gemm_mp_ctx *ctx);

/* Unpack [async]: the numbers the packed tiles stand for (stored value times 2^e), exactly,
 * as a dense FP64 device matrix.  For verification; not part of the timed path. */
int gemm_mp_unpack_tiles(gemm_mp_ctx *ctx, char which, double *dense_dev, int64_t ld,
                         gemm_mp_stream stream);

/* Descriptor of tile (I,J) of `which`: byte offset in the packed buffer, precision code and
 * scale exponent (each pointer may be NULL).  The exponent is known once the matrix has been
 * packed (or its map computed by the norm rule); asking for it earlier is ESTATE.  [sync on
 * the stream last used for that matrix when the exponent is requested] */
int gemm_mp_tile_info(gemm_mp_ctx *ctx, char which, int32_t I, int32_t J, size_t *offset,
                      int *prec, int *scale_exp);

/* Product and storage statistics of the current maps and policy; ESTATE until all three maps
 * are set.  Host only. */
int gemm_mp_get_stats(gemm_mp_ctx *ctx, gemm_mp_stats *out);

/* How often this context has allocated device or pinned host memory, and how often it has made the
 * host wait for the device, since it was created (either pointer may be NULL).  For callers and
 * tests that must know that a steady-state loop of pack / prepare / run does neither.  Host only. */
int gemm_mp_host_counters(gemm_mp_ctx *ctx, int64_t *allocations, int64_t *host_waits);

/* Product precision the given policy assigns (pure function; -1 on a bad code). */
int gemm_mp_product_precision(int pA, int pB, int pC, int policy);

/* Static, human-readable text for a status code. */
const char *gemm_mp_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* GEMM_MP_H */
