// Host side of libgemm_mp: context, precision maps, packed layout, the precision-bucketed
// owner-workgroup schedule, and the C ABI declared in include/gemm_mp.h.
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <numeric>
#include <vector>

#include "gemm_mp_internal.h"

using namespace gmp;

namespace {

// A small table that lives twice: in device memory, where the kernels read it, and in pinned host
// memory, where the host composes it and from where it is copied with hipMemcpyAsync on the
// caller's stream.  Both grow on demand and are never shrunk, so a context that sees the same
// shapes again allocates nothing.  The pinned half has two slots used in turn, each with an
// event that marks its last upload: the host rewrites a slot only after that upload has left,
// which it finds to be so without waiting unless it is two uploads ahead of the device.
template <typename T>
struct Mirror {
    T *dev = nullptr;
    T *pin[2] = {nullptr, nullptr};
    hipEvent_t sent[2] = {nullptr, nullptr};
    bool pending[2] = {false, false};
    int slot = 0;
    size_t cap = 0;
};

struct Matrix {
    int64_t rows = 0, cols = 0;    // entries of the dense matrix
    int rows_t = 0, cols_t = 0;    // tiles: ceil(rows / nb), ceil(cols / nb)
    bool transposed = false;       // dense buffers of this matrix hold its transpose (cols x rows)
    bool has_map = false;
    std::vector<uint16_t> map;
    std::vector<uint64_t> offset;
    uint64_t bytes = 0;
    void *storage = nullptr;
    size_t storage_bytes = 0;
    bool packed = false;
    bool exps_valid = false;       // device exponents describe the packed (or to-be-packed) data
    bool exps_from_rule = false;   // ... and were taken from the scan of the norm rule
    bool tables_current = false;   // device copies of prec / offset match the host map
    Mirror<uint8_t> prec;          // [tiles] precision codes
    Mirror<uint64_t> off;          // [tiles] byte offsets
    int32_t *d_exp = nullptr;
    double *d_sumsq = nullptr, *d_maxabs = nullptr, *d_part_sum = nullptr, *d_part_max = nullptr;
    // C only: the tiles stored in FP16 / FP8, each with an FP32 staging copy behind the packed
    // tiles; the offset table the GEMM kernels see points those tiles at their staging copies
    std::vector<LowTile> low;
    Mirror<LowTile> lowt;
    Mirror<uint64_t> off_run;
    float *d_low_max = nullptr;
    size_t low_max_cap = 0;
    hipStream_t last_stream = nullptr;
    int ntiles() const { return rows_t * cols_t; }
};

}  // namespace

struct gemm_mp_ctx {
    int64_t M, N, K;
    int nb, MT, NT, KT;
    int policy = GEMM_MP_POLICY_OPERAND;
    Matrix mat[3];
    bool sched_current = false;
    std::vector<uint8_t> q;
    std::vector<WorkItem> items[8];   // regions of [0] FP64 C tiles, [1] C tiles accumulated in FP32 (stored
                                      // FP32 / FP16 / FP8), [2] those of them whose products are all
                                      // FP8 x FP8 (256 x 256 regions), [3] / [4] the same for MXFP8 x MXFP8 / MXFP4 x MXFP4,
                                      // [5] / [6] for FP16 x FP16 / BF16 x BF16, [7] for MXFP6 x MXFP6
    Mirror<uint8_t> qd;               // [MT*NT][KT] product precision of every task
    Mirror<WorkItem> itemsd;          // the lists, [0] first
    ProductDesc *d_prod = nullptr;    // one record per task (+ 2 padding records), filled on the device
    size_t prod_cap = 0;
    bool sched_uploaded = false;      // the device copies of q and the lists are those of the current schedule
    hipStream_t sched_stream = nullptr;
    LaunchLanes lanes{};              // side streams of a run (made with the schedule's tables)
    bool has_lanes = false;
    bool serial = false;              // keep the launches of a run on the caller's stream, one after the other
    int64_t n_allocs = 0;             // device / pinned allocations this context has made
    int64_t n_syncs = 0;              // times it made the host wait for the device
    gemm_mp_stats stats;
    bool mixed32 = false;             // list [1] holds an FP16 / BF16 product with an operand stored in FP8
    bool mixed64 = false;             // the same for list [0]
    bool low64 = false;               // no region of list [0] has an FP64 product
    bool has_bf16 = false;            // some product of the 128 x 128 kernels has a BF16 or block-scaled operand
    bool kernel_ready = false;
    // sender-side conversion: per tile of A / B and product precision q, the offset of the copy
    // in precision q inside the workspace (kNoCopy: no task needs one)
    std::vector<uint64_t> conv_off[2];
    uint64_t conv_bytes = 0;
    int64_t conv_tiles = 0;
    bool conv_active = false;         // the workspace holds copies that match maps, policy and packed data
    uint64_t *d_conv[2] = {nullptr, nullptr};   // [tiles][8] device addresses of the copies, 0 = none
    ConvertJob *d_jobs = nullptr;
};

constexpr uint64_t kNoCopy = ~(uint64_t)0;

namespace {

int which_index(char w)
{
    switch (w) {
    case 'A': case 'a': return 0;
    case 'B': case 'b': return 1;
    case 'C': case 'c': return 2;
    default: return -1;
    }
}

#define HIP_TRY(expr) do { if ((expr) != hipSuccess) { (void)hipGetLastError(); return GEMM_MP_EHIP; } } while (0)

// Device allocation of a table that is made once and kept (n elements + padding for the aligned
// word reads of byte tables).
template <typename T>
int dev_alloc(gemm_mp_ctx *c, T **p, size_t n)
{
    if (*p) return GEMM_MP_OK;
    if (hipMalloc((void **)p, n * sizeof(T) + 16) != hipSuccess) { (void)hipGetLastError(); *p = nullptr; return GEMM_MP_ENOMEM; }
    c->n_allocs += 1;
    return GEMM_MP_OK;
}

// Room for n elements in both halves of a mirror.  Growing frees the old halves (hipFree waits
// for the device, so nothing still reads them).
template <typename T>
void release(Mirror<T> &m)
{
    (void)hipFree(m.dev);
    for (int k = 0; k < 2; ++k) {
        (void)hipHostFree(m.pin[k]);
        if (m.sent[k]) (void)hipEventDestroy(m.sent[k]);
        m.pin[k] = nullptr; m.sent[k] = nullptr; m.pending[k] = false;
    }
    m.dev = nullptr; m.cap = 0;
}
template <typename T>
int reserve(gemm_mp_ctx *c, Mirror<T> &m, size_t n)
{
    if (m.cap >= n && m.dev) return GEMM_MP_OK;
    release(m);
    bool ok = hipMalloc((void **)&m.dev, n * sizeof(T) + 16) == hipSuccess;
    for (int k = 0; ok && k < 2; ++k)
        ok = hipHostMalloc((void **)&m.pin[k], n * sizeof(T) + 16, hipHostMallocDefault) == hipSuccess &&
             hipEventCreateWithFlags(&m.sent[k], hipEventDisableTiming) == hipSuccess;
    if (!ok) { (void)hipGetLastError(); release(m); return GEMM_MP_ENOMEM; }
    c->n_allocs += 3;
    m.cap = n;
    return GEMM_MP_OK;
}
// The pinned slot the host may compose the next version of the table in (null on a HIP error).
template <typename T>
T *begin_write(gemm_mp_ctx *c, Mirror<T> &m)
{
    m.slot ^= 1;
    if (m.pending[m.slot]) {
        if (hipEventQuery(m.sent[m.slot]) != hipSuccess) {
            (void)hipGetLastError();
            if (hipEventSynchronize(m.sent[m.slot]) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
            c->n_syncs += 1;
        }
        m.pending[m.slot] = false;
    }
    return m.pin[m.slot];
}
// Queue the copy of the first n elements of that slot to the device half on stream s.
template <typename T>
int upload(Mirror<T> &m, size_t n, hipStream_t s)
{
    if (n) HIP_TRY(hipMemcpyAsync(m.dev, m.pin[m.slot], n * sizeof(T), hipMemcpyHostToDevice, s));
    HIP_TRY(hipEventRecord(m.sent[m.slot], s));
    m.pending[m.slot] = true;
    return GEMM_MP_OK;
}
int host_wait(gemm_mp_ctx *c, hipStream_t s)
{
    HIP_TRY(hipStreamSynchronize(s));
    c->n_syncs += 1;
    return GEMM_MP_OK;
}

void free_matrix_tables(Matrix &m)
{
    release(m.prec); release(m.off); release(m.lowt); release(m.off_run);
    (void)hipFree(m.d_exp);
    (void)hipFree(m.d_sumsq); (void)hipFree(m.d_maxabs); (void)hipFree(m.d_part_sum); (void)hipFree(m.d_part_max);
    (void)hipFree(m.d_low_max);
    m.d_low_max = nullptr; m.low_max_cap = 0;
    m.d_exp = nullptr;
    m.d_sumsq = m.d_maxabs = m.d_part_sum = m.d_part_max = nullptr;
}

// Packed layout: tiles in row-major order, each at a 256-byte aligned offset.  Behind the tiles
// of C follows one FP32 staging copy per tile stored in FP16 / FP8, in tile order.
void layout(gemm_mp_ctx *c, Matrix &m, bool is_c)
{
    const uint64_t elems = (uint64_t)c->nb * (uint64_t)c->nb;
    m.offset.resize(m.ntiles());
    uint64_t off = 0;
    for (int t = 0; t < m.ntiles(); ++t) {
        m.offset[t] = off;
        off += (tile_bytes_of(m.map[t], elems) + 255u) & ~(uint64_t)255u;
    }
    m.low.clear();
    for (int t = 0; is_c && t < m.ntiles(); ++t)
        if (m.map[t] >= GEMM_MP_FP16) {
            LowTile lt;
            lt.stage = off;
            lt.tile = (uint32_t)t;
            lt.pad = 0;
            m.low.push_back(lt);
            off += elems * sizeof(float);
        }
    m.bytes = off;
}

int install_map(gemm_mp_ctx *c, int w, const uint16_t *map)
{
    Matrix &m = c->mat[w];
    m.map.assign(map, map + m.ntiles());
    m.has_map = true;
    layout(c, m, w == 2);
    m.storage = nullptr;
    m.storage_bytes = 0;
    m.packed = false;
    m.exps_valid = false;
    m.exps_from_rule = false;
    m.tables_current = false;
    c->sched_current = false;
    c->sched_uploaded = false;
    return GEMM_MP_OK;
}

// Device copies of the per-tile tables (small; owned by the library), brought up to date with
// copies queued on stream s: later work on s sees them, and nothing here waits for the device
// once the tables have their size.
int ensure_tables(gemm_mp_ctx *c, Matrix &m, hipStream_t s)
{
    const size_t n = (size_t)m.ntiles();
    int rc;
    if ((rc = reserve(c, m.prec, n)) || (rc = reserve(c, m.off, n))) return rc;
    if (!m.d_exp) {
        if ((rc = dev_alloc(c, &m.d_exp, n))) return rc;
        HIP_TRY(hipMemsetAsync(m.d_exp, 0, n * sizeof(int32_t), s));
    }
    if (m.tables_current) return GEMM_MP_OK;
    if (!m.low.empty()) {
        const size_t elems = (size_t)((m.bytes - m.low[0].stage) / m.low.size() / sizeof(float));   // nb * nb
        const size_t need = m.low.size() * (elems / kLowChunk);
        if ((rc = reserve(c, m.lowt, n)) || (rc = reserve(c, m.off_run, n))) return rc;
        if (m.low_max_cap < need) {
            (void)hipFree(m.d_low_max);
            m.d_low_max = nullptr;
            m.low_max_cap = 0;
            if ((rc = dev_alloc(c, &m.d_low_max, need))) return rc;
            m.low_max_cap = need;
        }
    }
    uint8_t *p8 = begin_write(c, m.prec);
    uint64_t *po = begin_write(c, m.off);
    if (!p8 || !po) return GEMM_MP_EHIP;
    for (size_t t = 0; t < n; ++t) p8[t] = (uint8_t)m.map[t];
    std::memcpy(po, m.offset.data(), n * sizeof(uint64_t));
    if ((rc = upload(m.prec, n, s)) || (rc = upload(m.off, n, s))) return rc;
    if (!m.low.empty()) {
        uint64_t *pr = begin_write(c, m.off_run);
        LowTile *pl = begin_write(c, m.lowt);
        if (!pr || !pl) return GEMM_MP_EHIP;
        std::memcpy(pr, m.offset.data(), n * sizeof(uint64_t));
        for (const LowTile &lt : m.low) pr[lt.tile] = lt.stage;
        std::memcpy(pl, m.low.data(), m.low.size() * sizeof(LowTile));
        if ((rc = upload(m.lowt, m.low.size(), s)) || (rc = upload(m.off_run, n, s))) return rc;
    }
    m.tables_current = true;
    return GEMM_MP_OK;
}

int ensure_scan_buffers(gemm_mp_ctx *c, Matrix &m)
{
    const size_t n = (size_t)m.ntiles(), parts = (size_t)(c->nb / kScanCols);
    int rc;
    if ((rc = dev_alloc(c, &m.d_sumsq, n))) return rc;
    if ((rc = dev_alloc(c, &m.d_maxabs, n))) return rc;
    if ((rc = dev_alloc(c, &m.d_part_sum, n * parts))) return rc;
    if ((rc = dev_alloc(c, &m.d_part_max, n * parts))) return rc;
    return GEMM_MP_OK;
}

PackedView view_of(const Matrix &m)
{
    PackedView v;
    v.prec = m.prec.dev;
    v.offset = m.off.dev;
    v.exp = m.d_exp;
    v.storage = (char *)m.storage;
    return v;
}

int check_dense(const void *p, int64_t ld, int64_t cols)
{
    if (!p || ld < cols || (ld & 1) || ((uintptr_t)p & 15u)) return GEMM_MP_EINVAL;
    return GEMM_MP_OK;
}

double unit_roundoff(int p)
{
    static const double u[7] = {0x1p-53, 0x1p-24, 0x1p-11, 0x1p-4, 0x1p-8, 0x1p-4, 0x1p-2};
    return u[p];
}

// Relative cost of one tile product by precision: inverse matrix-core peak (FP64 : FP32 :
// FP16 : FP8 = 1/78.6 : 1/157.3 : 1/2516.6 : 1/5033.2 TFLOP/s) plus a floor for the operand
// traffic that the low precisions cannot hide.
const double kCost[8] = {64.0, 32.0, 3.0, 2.0, 3.0, 2.0, 1.5, 2.0};

// The schedule.  Every C tile is cut into (nb/128)^2 owner regions; a region's cost is the
// sum over its reduction tiles of the cost of that product's precision.  C tiles are sorted by
// cost, dealt to eight bins (one per XCD: workgroup p is dispatched to XCD p mod 8) so that the
// bins' total costs are balanced, heaviest first; the launch order interleaves the bins, so
// each XCD works through its own C tiles, keeping their A row panels and B column panels in
// its L2, and the cheap regions fill the tail.
void build_schedule(gemm_mp_ctx *c)
{
    const int MT = c->MT, NT = c->NT, KT = c->KT;
    const Matrix &A = c->mat[0], &B = c->mat[1], &C = c->mat[2];
    c->q.resize((size_t)MT * NT * KT);
    std::memset(&c->stats, 0, sizeof(c->stats));
    std::vector<double> cost((size_t)MT * NT, 0.0);
    for (int I = 0; I < MT; ++I)
        for (int J = 0; J < NT; ++J) {
            const int pC = C.map[I * NT + J];
            for (int L = 0; L < KT; ++L) {
                const int q = product_precision(A.map[I * KT + L], B.map[L * NT + J], pC, c->policy);
                c->q[((size_t)I * NT + J) * KT + L] = (uint8_t)q;
                if (q == GEMM_MP_BF16) c->stats.products_bf16 += 1;
                else if (q == GEMM_MP_MXFP8) c->stats.products_mxfp8 += 1;
                else if (q == GEMM_MP_MXFP4) c->stats.products_mxfp4 += 1;
                else if (q == GEMM_MP_MXFP6) c->stats.products_mxfp6 += 1;
                else c->stats.products[q] += 1;
                cost[(size_t)I * NT + J] += kCost[q];
            }
        }
    const double f = 2.0 * (double)c->nb * (double)c->nb * (double)c->nb;
    for (int q = 0; q < 4; ++q) c->stats.flops[q] = f * (double)c->stats.products[q];
    c->stats.flops_bf16 = f * (double)c->stats.products_bf16;
    c->stats.flops_mxfp8 = f * (double)c->stats.products_mxfp8;
    c->stats.flops_mxfp4 = f * (double)c->stats.products_mxfp4;
    c->stats.flops_mxfp6 = f * (double)c->stats.products_mxfp6;

    // A C tile accumulated in FP32 whose every product multiplies two MXFP8 tiles goes to the
    // block-scaled instance of the 256 x 256 kernel.  Every other product with an MXFP8 operand
    // is run by the 128 x 128 kernels, which widen the block-scaled tiles on the receiving side
    // (element times block scale, exact) or read the sender-side copies where there are any:
    // at FP32 where both operands are MXFP8 (exact products, FP32 accumulation: what an MXFP8
    // product is), at the product's own FP32 / FP64 otherwise.  c->q then holds the precision
    // the kernels work at, the statistics keep the product's nominal one.
    std::vector<uint8_t> all_mx((size_t)MT * NT, 0);         // 1: all MXFP8 x MXFP8, 2: all MXFP4 x MXFP4 (tile size a multiple of 512), 3: all MXFP6 x MXFP6
    for (int I = 0; I < MT; ++I)
        for (int J = 0; J < NT; ++J) {
            const bool fits = C.map[I * NT + J] != GEMM_MP_FP64 && KT > 0;
            bool all8 = fits && c->nb % kMacroFp8 == 0, all4 = fits && c->nb % (2 * kMacroFp8) == 0, all6 = all8;
            for (int L = 0; L < KT; ++L) {
                all8 &= c->q[((size_t)I * NT + J) * KT + L] == GEMM_MP_MXFP8;
                all4 &= c->q[((size_t)I * NT + J) * KT + L] == GEMM_MP_MXFP4;
                all6 &= c->q[((size_t)I * NT + J) * KT + L] == GEMM_MP_MXFP6;
            }
            all_mx[(size_t)I * NT + J] = all8 ? 1 : all4 ? 2 : all6 ? 3 : 0;
            if (!all8 && !all4 && !all6)
                for (int L = 0; L < KT; ++L) {
                    uint8_t &q = c->q[((size_t)I * NT + J) * KT + L];
                    if (is_block_scaled(q)) q = GEMM_MP_FP32;
                }
        }

    // Sender-side conversion plan: which (tile, q) copies the tasks would need, and where each
    // would live in the workspace (256-byte aligned, A's copies first).
    c->conv_off[0].assign((size_t)MT * KT * kConvSlots, kNoCopy);
    c->conv_off[1].assign((size_t)KT * NT * kConvSlots, kNoCopy);
    for (int I = 0; I < MT; ++I)
        for (int J = 0; J < NT; ++J)
            for (int L = 0; L < KT; ++L) {
                const int q = c->q[((size_t)I * NT + J) * KT + L];
                const int pa = A.map[I * KT + L], pb = B.map[L * NT + J];
                if (is_block_scaled(q)) continue;                             // block-scaled kernel: no copies
                if (pa != q) c->conv_off[0][((size_t)I * KT + L) * kConvSlots + q] = 0;
                if (pb != q) c->conv_off[1][((size_t)L * NT + J) * kConvSlots + q] = 0;
            }
    c->conv_bytes = 0;
    c->conv_tiles = 0;
    for (int w = 0; w < 2; ++w)
        for (size_t k = 0; k < c->conv_off[w].size(); ++k)
            if (c->conv_off[w][k] != kNoCopy) {
                const int q = (int)(k % kConvSlots);
                c->conv_off[w][k] = c->conv_bytes;
                c->conv_bytes += (((uint64_t)c->nb * c->nb * elem_bytes(q)) + 255) & ~(uint64_t)255;
                c->conv_tiles += 1;
            }
    c->conv_active = false;
    for (int w = 0; w < 3; ++w) {
        for (int t = 0; t < c->mat[w].ntiles(); ++t) {
            const int p = c->mat[w].map[t];
            if (p == GEMM_MP_BF16) c->stats.tiles_bf16[w] += 1;
            else if (p == GEMM_MP_MXFP8) c->stats.tiles_mxfp8[w] += 1;
            else if (p == GEMM_MP_MXFP4) c->stats.tiles_mxfp4[w] += 1;
            else if (p == GEMM_MP_MXFP6) c->stats.tiles_mxfp6[w] += 1;
            else c->stats.tiles[w][p] += 1;
        }
        c->stats.packed_bytes[w] = c->mat[w].bytes;
    }

    // A C tile accumulated in FP32 whose every product multiplies two tiles stored in FP8 at FP8
    // goes to the kernel with 256 x 256 regions (the tile size permitting).
    std::vector<uint8_t> all_fp8((size_t)MT * NT, 0);
    if (c->nb % kMacroFp8 == 0)
        for (int I = 0; I < MT; ++I)
            for (int J = 0; J < NT; ++J) {
                bool ok = C.map[I * NT + J] != GEMM_MP_FP64 && KT > 0;
                for (int L = 0; ok && L < KT; ++L)
                    ok = c->q[((size_t)I * NT + J) * KT + L] == GEMM_MP_FP8_E4M3 && A.map[I * KT + L] == GEMM_MP_FP8_E4M3 &&
                         B.map[L * NT + J] == GEMM_MP_FP8_E4M3;
                all_fp8[(size_t)I * NT + J] = ok;
            }
    // ... and likewise a tile whose every product multiplies two FP16 tiles, or two BF16 tiles (the
    // 32x32x16 matrix instructions; the FP16 tiles' scales are followed by rescaling the sums)
    std::vector<uint8_t> all_16((size_t)MT * NT, 0);         // 1: all FP16 x FP16, 2: all BF16 x BF16
    if (c->nb % kMacroFp8 == 0)
        for (int I = 0; I < MT; ++I)
            for (int J = 0; J < NT; ++J) {
                bool h = C.map[I * NT + J] != GEMM_MP_FP64 && KT > 0, b = h;
                for (int L = 0; (h || b) && L < KT; ++L) {
                    const int q = c->q[((size_t)I * NT + J) * KT + L], pa = A.map[I * KT + L], pb = B.map[L * NT + J];
                    h = h && q == GEMM_MP_FP16 && pa == GEMM_MP_FP16 && pb == GEMM_MP_FP16;
                    b = b && q == GEMM_MP_BF16 && pa == GEMM_MP_BF16 && pb == GEMM_MP_BF16;
                }
                all_16[(size_t)I * NT + J] = h ? 1 : b ? 2 : 0;
            }
    // The formats beyond FP64 / FP32 / FP16 / FP8 (BF16 products in the ring, BF16 and block-scaled
    // tiles widened under FP32 / FP64 products) are known to one instance of the 128 x 128 kernel
    // only; it serves both launches as soon as one product of theirs has such an operand.
    c->mixed32 = c->mixed64 = c->has_bf16 = false;
    c->low64 = true;                                     // no FP64 C tile has an FP64 product
    for (int I = 0; I < MT; ++I)
        for (int J = 0; J < NT; ++J) {
            if (all_fp8[(size_t)I * NT + J] || all_16[(size_t)I * NT + J] || all_mx[(size_t)I * NT + J]) continue;
            bool mixed = false;
            for (int L = 0; L < KT; ++L) {
                const int q = c->q[((size_t)I * NT + J) * KT + L];
                const int pa = A.map[I * KT + L], pb = B.map[L * NT + J];
                c->has_bf16 |= pa == GEMM_MP_BF16 || pb == GEMM_MP_BF16 || is_block_scaled(pa) || is_block_scaled(pb);
                mixed |= (q == GEMM_MP_FP16 || q == GEMM_MP_BF16) &&
                         (A.map[I * KT + L] == GEMM_MP_FP8_E4M3 || B.map[L * NT + J] == GEMM_MP_FP8_E4M3);
            }
            if (C.map[I * NT + J] == GEMM_MP_FP64) c->mixed64 |= mixed;
            else c->mixed32 |= mixed;
            if (C.map[I * NT + J] == GEMM_MP_FP64)
                for (int L = 0; L < KT; ++L) c->low64 &= c->q[((size_t)I * NT + J) * KT + L] != GEMM_MP_FP64;
        }
    constexpr int kBins = 8;
    for (int list = 0; list < 8; ++list) {
        const int mr = c->nb / (list >= 2 ? kMacroFp8 : kMacro);
        const size_t per_tile = (size_t)mr * mr;
        std::vector<WorkItem> bins[kBins];
        {
            // C tiles sorted by cost and dealt to the bins, heaviest first; a tile's regions stay
            // together.  (For the 256 x 256 regions, whose kernels wait for operand bytes, an order
            // in which the 32 regions an XCD holds at a time form a compact 4 x 8 block of C across
            // two tiles was measured too: same run time, more bytes fetched into the L2s.)
            std::vector<int> order;
            for (int t = 0; t < MT * NT; ++t) {
                const int which = C.map[t] == GEMM_MP_FP64 ? 0 : all_fp8[t] ? 2 : all_mx[t] == 3 ? 7 : all_mx[t] ? 2 + all_mx[t] : all_16[t] ? 4 + all_16[t] : 1;
                if (which == list) order.push_back(t);
            }
            std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return cost[a] > cost[b]; });
            double load[kBins] = {0};
            for (int t : order) {
                int best = 0;
                for (int b = 1; b < kBins; ++b)
                    if (load[b] < load[best]) best = b;
                load[best] += cost[t];
                // the 32 regions of a tile that an XCD works on at a time: a 4 x 8 block of the tile
                // where its regions form more than 8 columns (they read 4 + 8 strips of the operand
                // panels through that XCD's L2 instead of 2 + 16 or 1 + 32), else row by row
                const bool blocked = list < 2 && mr > 8 && mr % 8 == 0;
                for (size_t r = 0; r < per_tile; ++r) {
                    WorkItem it;
                    it.tile = (uint32_t)t;
                    if (blocked) {
                        const int blk = (int)(r / 32), in = (int)(r % 32), bpr = mr / 8;      // blocks per block row
                        it.mi = (uint16_t)((blk / bpr) * 4 + in / 8);
                        it.mj = (uint16_t)((blk % bpr) * 8 + in % 8);
                    } else {
                        it.mi = (uint16_t)(r / mr);
                        it.mj = (uint16_t)(r % mr);
                    }
                    bins[best].push_back(it);
                }
            }
        }
        // launch order: the bins interleaved, workgroup p landing on XCD p mod 8
        std::vector<WorkItem> &items = c->items[list];
        items.clear();
        size_t pos[kBins] = {0};
        bool any = true;
        while (any) {
            any = false;
            for (int b = 0; b < kBins; ++b) {
                if (pos[b] >= bins[b].size()) continue;
                any = true;
                items.push_back(bins[b][pos[b]++]);
            }
        }
    }
    c->stats.work_items = 0;
    for (int list = 0; list < 8; ++list) {
        c->stats.launch_items[list] = (int64_t)c->items[list].size();
        c->stats.work_items += (int64_t)c->items[list].size();
    }
    c->stats.owner_instance[0] = c->has_bf16 ? 2 : c->mixed64 ? 1 : c->low64 ? 3 : 0;
    c->stats.owner_instance[1] = c->has_bf16 ? 2 : c->mixed32 ? 1 : 0;
    c->sched_current = true;
}

// The schedule of the current maps and policy on the device: built on the host if it is not
// current, composed in pinned memory and copied with hipMemcpyAsync on stream s.  The device
// tables are sized for the largest schedule these shapes can have, so a context allocates them
// once.
int prepare_schedule(gemm_mp_ctx *c, hipStream_t s)
{
    if (!c->sched_current) build_schedule(c);
    if (c->sched_uploaded) return GEMM_MP_OK;
    if (!c->has_lanes) {
        for (int k = 0; k < 4; ++k) {
            HIP_TRY(hipStreamCreateWithFlags(&c->lanes.side[k], hipStreamNonBlocking));
            HIP_TRY(hipEventCreateWithFlags(&c->lanes.join[k], hipEventDisableTiming));
        }
        HIP_TRY(hipEventCreateWithFlags(&c->lanes.fork, hipEventDisableTiming));
        c->has_lanes = true;
        c->n_allocs += 1;
    }
    const size_t tasks = c->q.size();
    const size_t per_tile = (size_t)(c->nb / kMacro) * (size_t)(c->nb / kMacro);
    const size_t max_items = (size_t)c->MT * c->NT * per_tile;
    int rc;
    if ((rc = reserve(c, c->qd, tasks)) || (rc = reserve(c, c->itemsd, max_items))) return rc;
    if (c->prod_cap < tasks + 2) {
        (void)hipFree(c->d_prod);
        c->d_prod = nullptr;
        c->prod_cap = 0;
        if ((rc = dev_alloc(c, &c->d_prod, tasks + 2))) return rc;
        c->prod_cap = tasks + 2;
        HIP_TRY(hipMemsetAsync(c->d_prod, 0, (tasks + 2) * sizeof(ProductDesc), s));
    }
    uint8_t *pq = begin_write(c, c->qd);
    WorkItem *pi = begin_write(c, c->itemsd);
    if (!pq || !pi) return GEMM_MP_EHIP;
    std::memcpy(pq, c->q.data(), tasks);
    size_t n = 0;
    for (int list = 0; list < 8; ++list) {
        if (!c->items[list].empty()) std::memcpy(pi + n, c->items[list].data(), c->items[list].size() * sizeof(WorkItem));
        n += c->items[list].size();
    }
    if ((rc = upload(c->qd, tasks, s)) || (rc = upload(c->itemsd, n, s))) return rc;
    c->sched_uploaded = true;
    c->sched_stream = s;
    return GEMM_MP_OK;
}

bool all_maps(const gemm_mp_ctx *c) { return c->mat[0].has_map && c->mat[1].has_map && c->mat[2].has_map; }

int run_scan(gemm_mp_ctx *c, Matrix &m, const double *dense, int64_t ld, hipStream_t s)
{
    int rc;
    if ((rc = ensure_scan_buffers(c, m))) return rc;
    HIP_TRY(launch_scan(dense, ld, m.transposed, m.rows, m.cols, m.rows_t, m.cols_t, c->nb, m.d_part_sum, m.d_part_max, m.d_sumsq, m.d_maxabs, s));
    return GEMM_MP_OK;
}

// ---- scratch of gemm_mp_run_static -----------------------------------------------------------
// The product table of a run (one 32-byte record per tile product, written by a small kernel
// before the GEMM kernels read it) is the one piece of scratch memory gemm_mp_run takes from an
// allocation of its own.  The entry point that must not allocate keeps it here instead: a
// file-scope device array, one copy per GPU, held until the process ends.  In host code the
// array's name is only a handle: the address a kernel can use comes from hipGetSymbolAddress,
// asked once per device with that device current, and only that address is passed on.
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[((size_t)GEMM_MP_STATIC_MAX_PRODUCTS + 2) * sizeof(ProductDesc)];
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_lock;

// out == nullptr: only make sure the current device's address is known.
int static_scratch(ProductDesc **out)
{
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return GEMM_MP_EHIP;
    std::lock_guard<std::mutex> guard(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return GEMM_MP_EHIP;
        g_scratch_ptr[dev] = p;
    }
    if (out) *out = (ProductDesc *)g_scratch_ptr[dev];
    return GEMM_MP_OK;
}

}  // namespace

extern "C" {

int gemm_mp_create(gemm_mp_ctx **out, int64_t M, int64_t N, int64_t K, int32_t nb)
{
    if (!out || M <= 0 || N <= 0 || K <= 0 || nb <= 0) return GEMM_MP_EINVAL;
    if (nb % kMacro != 0 || nb > 8192) return GEMM_MP_EINVAL;
    const int64_t mt = (M + nb - 1) / nb, nt = (N + nb - 1) / nb, kt = (K + nb - 1) / nb;
    if (mt > 32767 || nt > 32767 || kt > 32767) return GEMM_MP_EINVAL;
    if (mt * nt > (int64_t)1 << 24 || mt * nt * kt > (int64_t)1 << 28) return GEMM_MP_EINVAL;
    // pack and unpack put 64-row blocks of a matrix into the second grid dimension (at most 65535)
    if (mt * nb / kPackBlock > 65535 || nt * nb / kPackBlock > 65535 || kt * nb / kPackBlock > 65535) return GEMM_MP_EINVAL;
    gemm_mp_ctx *c = new (std::nothrow) gemm_mp_ctx();
    if (!c) return GEMM_MP_ENOMEM;
    c->M = M; c->N = N; c->K = K; c->nb = nb;
    c->MT = (int)mt; c->NT = (int)nt; c->KT = (int)kt;
    c->mat[0].rows_t = c->MT; c->mat[0].cols_t = c->KT; c->mat[0].rows = M; c->mat[0].cols = K;
    c->mat[1].rows_t = c->KT; c->mat[1].cols_t = c->NT; c->mat[1].rows = K; c->mat[1].cols = N;
    c->mat[2].rows_t = c->MT; c->mat[2].cols_t = c->NT; c->mat[2].rows = M; c->mat[2].cols = N;
    std::memset(&c->stats, 0, sizeof(c->stats));
    const char *serial = std::getenv("GEMM_MP_SERIAL_LAUNCHES");
    c->serial = serial && serial[0] == '1';
    *out = c;
    return GEMM_MP_OK;
}

int gemm_mp_destroy(gemm_mp_ctx *c)
{
    if (!c) return GEMM_MP_EINVAL;
    for (auto &m : c->mat) free_matrix_tables(m);
    release(c->qd); release(c->itemsd);
    (void)hipFree(c->d_prod);
    if (c->has_lanes) {
        for (int k = 0; k < 4; ++k) { (void)hipStreamDestroy(c->lanes.side[k]); (void)hipEventDestroy(c->lanes.join[k]); }
        (void)hipEventDestroy(c->lanes.fork);
    }
    (void)hipFree(c->d_conv[0]); (void)hipFree(c->d_conv[1]); (void)hipFree(c->d_jobs);

    (void)hipGetLastError();
    delete c;
    return GEMM_MP_OK;
}

int gemm_mp_set_policy(gemm_mp_ctx *c, int policy)
{
    if (!c || (policy != GEMM_MP_POLICY_OPERAND && policy != GEMM_MP_POLICY_C_TILE)) return GEMM_MP_EINVAL;
    if (policy != c->policy) { c->policy = policy; c->sched_current = false; c->sched_uploaded = false; }
    return GEMM_MP_OK;
}

int gemm_mp_set_transposed(gemm_mp_ctx *c, char which, int transposed)
{
    const int w = which_index(which);
    if (!c || w < 0 || w == 2 || (transposed != 0 && transposed != 1)) return GEMM_MP_EINVAL;
    Matrix &m = c->mat[w];
    if (m.transposed != (transposed != 0)) {
        m.transposed = transposed != 0;
        m.exps_from_rule = false;                  // a scan made under the other layout says nothing now
    }
    return GEMM_MP_OK;
}

int gemm_mp_set_precision_map(gemm_mp_ctx *c, char which, const uint16_t *map, int32_t rows, int32_t cols)
{
    const int w = which_index(which);
    if (!c || w < 0 || !map) return GEMM_MP_EINVAL;
    Matrix &m = c->mat[w];
    if (rows != m.rows_t || cols != m.cols_t) return GEMM_MP_EINVAL;
    for (int t = 0; t < m.ntiles(); ++t)
        if (map[t] > GEMM_MP_MXFP6) return GEMM_MP_EINVAL;
    return install_map(c, w, map);
}

int gemm_mp_tile_scan(gemm_mp_ctx *c, char which, const double *dense, int64_t ld, gemm_mp_stream stream,
                      double *sumsq_host, double *maxabs_host)
{
    const int w = which_index(which);
    if (!c || w < 0) return GEMM_MP_EINVAL;
    Matrix &m = c->mat[w];
    int rc;
    if ((rc = check_dense(dense, ld, m.transposed ? m.rows : m.cols))) return rc;
    hipStream_t s = (hipStream_t)stream;
    if ((rc = run_scan(c, m, dense, ld, s))) return rc;
    if ((rc = host_wait(c, s))) return rc;
    const size_t n = (size_t)m.ntiles() * sizeof(double);
    if (sumsq_host) HIP_TRY(hipMemcpy(sumsq_host, m.d_sumsq, n, hipMemcpyDeviceToHost));
    if (maxabs_host) HIP_TRY(hipMemcpy(maxabs_host, m.d_maxabs, n, hipMemcpyDeviceToHost));
    m.exps_from_rule = false;     // the scan buffers no longer belong to a rule-made map
    return GEMM_MP_OK;
}

int gemm_mp_compute_precision_map(gemm_mp_ctx *c, char which, const double *dense, int64_t ld, double threshold,
                                  uint32_t allowed_mask, gemm_mp_stream stream, uint16_t *map_out)
{
    const int w = which_index(which);
    if (!c || w < 0 || !(threshold >= 0.0) || (allowed_mask & 0x1Fu) == 0 || (allowed_mask & ~0x1Fu)) return GEMM_MP_EINVAL;
    Matrix &m = c->mat[w];
    int rc;
    if ((rc = check_dense(dense, ld, m.transposed ? m.rows : m.cols))) return rc;
    hipStream_t s = (hipStream_t)stream;
    if ((rc = run_scan(c, m, dense, ld, s))) return rc;
    if ((rc = host_wait(c, s))) return rc;
    const int n = m.ntiles();
    std::vector<double> sumsq(n);
    HIP_TRY(hipMemcpy(sumsq.data(), m.d_sumsq, (size_t)n * sizeof(double), hipMemcpyDeviceToHost));

    // the rule, on squares, in a fixed order of operations (see the header)
    double S = 0.0;
    for (int t = 0; t < n; ++t) S = S + sumsq[t];
    const double rhs = (threshold * threshold) * S;
    static const int from_lowest[5] = {GEMM_MP_FP8_E4M3, GEMM_MP_BF16, GEMM_MP_FP16, GEMM_MP_FP32, GEMM_MP_FP64};
    int highest = GEMM_MP_FP64;
    for (int k = 0; k < 5; ++k)
        if (allowed_mask & (1u << from_lowest[k])) highest = from_lowest[k];
    std::vector<uint16_t> map(n);
    for (int t = 0; t < n; ++t) {
        int chosen = highest;
        for (int k = 0; k < 5; ++k) {
            const int p = from_lowest[k];
            if (!(allowed_mask & (1u << p))) continue;
            const double u = unit_roundoff(p);
            const double lhs = (sumsq[t] * (double)n) * (u * u);
            if (lhs <= rhs) { chosen = p; break; }
        }
        map[t] = (uint16_t)chosen;
    }
    if ((rc = install_map(c, w, map.data()))) return rc;
    if ((rc = ensure_tables(c, m, s))) return rc;
    HIP_TRY(launch_exps(m.d_maxabs, m.prec.dev, m.d_exp, n, s));
    m.exps_valid = true;
    m.exps_from_rule = true;
    m.last_stream = s;
    if (map_out) std::memcpy(map_out, map.data(), (size_t)n * sizeof(uint16_t));
    return GEMM_MP_OK;
}

int gemm_mp_storage_bytes(gemm_mp_ctx *c, char which, size_t *bytes)
{
    const int w = which_index(which);
    if (!c || w < 0 || !bytes) return GEMM_MP_EINVAL;
    if (!c->mat[w].has_map) return GEMM_MP_ESTATE;
    *bytes = (size_t)c->mat[w].bytes;
    return GEMM_MP_OK;
}

int gemm_mp_bind_storage(gemm_mp_ctx *c, char which, void *dev_ptr, size_t bytes)
{
    const int w = which_index(which);
    if (!c || w < 0 || !dev_ptr || ((uintptr_t)dev_ptr & 255u)) return GEMM_MP_EINVAL;
    Matrix &m = c->mat[w];
    if (!m.has_map) return GEMM_MP_ESTATE;
    if (bytes < m.bytes) return GEMM_MP_EINVAL;
    m.storage = dev_ptr;
    m.storage_bytes = bytes;
    m.packed = false;
    return GEMM_MP_OK;
}

int gemm_mp_pack_tiles(gemm_mp_ctx *c, char which, const double *dense, int64_t ld, gemm_mp_stream stream)
{
    const int w = which_index(which);
    if (!c || w < 0) return GEMM_MP_EINVAL;
    Matrix &m = c->mat[w];
    if (!m.has_map || !m.storage) return GEMM_MP_ESTATE;
    int rc;
    if ((rc = check_dense(dense, ld, m.transposed ? m.rows : m.cols))) return rc;
    hipStream_t s = (hipStream_t)stream;
    if ((rc = ensure_tables(c, m, s))) return rc;
    if (!m.exps_from_rule) {
        bool low = false;
        for (uint16_t p : m.map) low |= p == GEMM_MP_FP16 || p == GEMM_MP_FP8_E4M3;
        if (low) {
            if ((rc = run_scan(c, m, dense, ld, s))) return rc;
        } else if ((rc = ensure_scan_buffers(c, m))) return rc;
        HIP_TRY(launch_exps(m.d_maxabs, m.prec.dev, m.d_exp, m.ntiles(), s));
        m.exps_valid = true;
    }
    if (m.transposed)
        HIP_TRY(launch_pack(dense, ld, m.cols, m.rows, m.cols_t, m.rows_t, c->nb, w != 1, true, view_of(m), s));
    else
        HIP_TRY(launch_pack(dense, ld, m.rows, m.cols, m.rows_t, m.cols_t, c->nb, w == 1, false, view_of(m), s));
    bool has_mx = false;
    for (uint16_t p : m.map) has_mx |= is_block_scaled(p);
    if (has_mx)
        HIP_TRY(launch_pack_mx(dense, m.transposed ? 1 : ld, m.transposed ? ld : 1, m.rows, m.cols, m.rows_t, m.cols_t, c->nb, w == 1,
                               view_of(m), s));
    m.packed = true;
    m.last_stream = s;
    if (w < 2) c->conv_active = false;            // converted copies of the old data are stale
    return GEMM_MP_OK;
}

int gemm_mp_unpack_tiles(gemm_mp_ctx *c, char which, double *dense, int64_t ld, gemm_mp_stream stream)
{
    const int w = which_index(which);
    if (!c || w < 0) return GEMM_MP_EINVAL;
    Matrix &m = c->mat[w];
    if (!m.has_map || !m.storage) return GEMM_MP_ESTATE;
    int rc;
    if ((rc = check_dense(dense, ld, m.transposed ? m.rows : m.cols))) return rc;
    hipStream_t s = (hipStream_t)stream;
    if ((rc = ensure_tables(c, m, s))) return rc;
    if (m.transposed)
        HIP_TRY(launch_unpack(dense, ld, m.cols, m.rows, m.cols_t, m.rows_t, c->nb, w != 1, true, view_of(m), s));
    else
        HIP_TRY(launch_unpack(dense, ld, m.rows, m.cols, m.rows_t, m.cols_t, c->nb, w == 1, false, view_of(m), s));
    m.last_stream = s;
    return GEMM_MP_OK;
}

int gemm_mp_prepare(gemm_mp_ctx *c, gemm_mp_stream stream)
{
    if (!c) return GEMM_MP_EINVAL;
    if (!all_maps(c)) return GEMM_MP_ESTATE;
    hipStream_t s = (hipStream_t)stream;
    int rc;
    if ((rc = prepare_schedule(c, s))) return rc;
    if ((rc = ensure_tables(c, c->mat[2], s))) return rc;
    if (!c->kernel_ready) {
        HIP_TRY(gemm_kernel_setup());
        c->kernel_ready = true;
    }
    return static_scratch(nullptr);       // the current device's address of the static scratch, looked up once
}

namespace {

// What both forms of the run share.  prod: where the product table of this run is written.
int run_on(gemm_mp_ctx *c, double alpha, double beta, hipStream_t s, ProductDesc *prod)
{
    Matrix &A = c->mat[0], &B = c->mat[1], &C = c->mat[2];
    GemmArgs a;
    a.A = view_of(A); a.B = view_of(B); a.C = view_of(C);
    const int n_low = (int)C.low.size();
    if (n_low) {
        // FP16 / FP8 C tiles: the kernels work on the FP32 staging copies
        if (beta != 0.0) HIP_TRY(launch_low_expand(C.lowt.dev, n_low, c->nb, a.C, s));
        a.C.offset = C.off_run.dev;
    }
    a.q = c->qd.dev;
    a.prod = prod;
    a.convA = c->conv_active ? c->d_conv[0] : nullptr;
    a.convB = c->conv_active ? c->d_conv[1] : nullptr;
    a.items64 = c->itemsd.dev;
    a.items32 = a.items64 + c->items[0].size();
    a.items8 = a.items32 + c->items[1].size();
    a.n_items64 = (int32_t)c->items[0].size();
    a.n_items32 = (int32_t)c->items[1].size();
    a.n_items8 = (int32_t)c->items[2].size();
    a.items_mx = a.items8 + c->items[2].size();
    a.n_items_mx = (int32_t)c->items[3].size();
    a.items_mx4 = a.items_mx + c->items[3].size();
    a.n_items_mx4 = (int32_t)c->items[4].size();
    a.items_h = a.items_mx4 + c->items[4].size();
    a.n_items_h = (int32_t)c->items[5].size();
    a.items_bf = a.items_h + c->items[5].size();
    a.n_items_bf = (int32_t)c->items[6].size();
    a.items_mx6 = a.items_bf + c->items[6].size();
    a.n_items_mx6 = (int32_t)c->items[7].size();
    a.mixed32 = c->mixed32 ? 1 : 0;
    a.mixed64 = c->mixed64 ? 1 : 0;
    a.bf16 = c->has_bf16 ? 1 : 0;
    a.low64 = c->low64 ? 1 : 0;
    a.nb = c->nb; a.MT = c->MT; a.NT = c->NT; a.KT = c->KT;
    a.kt_eff = alpha == 0.0 ? 0 : c->KT;
    a.alpha = alpha; a.beta = beta;
    HIP_TRY(launch_gemm(a, s, c->has_lanes && !c->serial ? &c->lanes : nullptr));
    if (n_low) HIP_TRY(launch_low_store(C.lowt.dev, n_low, c->nb, view_of(C), C.d_exp, C.d_low_max, s));
    C.packed = true;
    C.exps_valid = true;
    A.last_stream = B.last_stream = C.last_stream = s;
    return GEMM_MP_OK;
}

int run_ready(gemm_mp_ctx *c, double alpha, double beta)
{
    if (!c || std::isnan(alpha) || std::isnan(beta)) return GEMM_MP_EINVAL;
    Matrix &A = c->mat[0], &B = c->mat[1], &C = c->mat[2];
    if (!all_maps(c) || !A.packed || !B.packed || !C.storage) return GEMM_MP_ESTATE;
    if (beta != 0.0 && !C.packed) return GEMM_MP_ESTATE;
    return GEMM_MP_OK;
}

}  // namespace

int gemm_mp_run(gemm_mp_ctx *c, double alpha, double beta, gemm_mp_stream stream)
{
    int rc;
    if ((rc = run_ready(c, alpha, beta))) return rc;
    if (!c->sched_current) build_schedule(c);
    hipStream_t s = (hipStream_t)stream;
    // what gemm_mp_prepare does, unless it has been done for these maps: only copies queued on s
    if ((rc = prepare_schedule(c, s))) return rc;
    if ((rc = ensure_tables(c, c->mat[2], s))) return rc;
    if (!c->kernel_ready) {
        HIP_TRY(gemm_kernel_setup());
        c->kernel_ready = true;
    }
    return run_on(c, alpha, beta, s, c->d_prod);
}

int gemm_mp_run_static(gemm_mp_ctx *c, double alpha, double beta, gemm_mp_stream stream)
{
    if (!c) return GEMM_MP_EINVAL;
    if ((int64_t)c->MT * c->NT * c->KT > (int64_t)GEMM_MP_STATIC_MAX_PRODUCTS) return GEMM_MP_ETOOBIG;
    int rc;
    if ((rc = run_ready(c, alpha, beta))) return rc;
    // everything that would allocate, build or copy must have happened in gemm_mp_prepare
    if (!c->sched_current || !c->sched_uploaded || !c->mat[2].tables_current || !c->kernel_ready) return GEMM_MP_ESTATE;
    ProductDesc *prod = nullptr;
    if ((rc = static_scratch(&prod))) return rc;
    return run_on(c, alpha, beta, (hipStream_t)stream, prod);
}

int gemm_mp_host_counters(gemm_mp_ctx *c, int64_t *allocations, int64_t *host_waits)
{
    if (!c) return GEMM_MP_EINVAL;
    if (allocations) *allocations = c->n_allocs;
    if (host_waits) *host_waits = c->n_syncs;
    return GEMM_MP_OK;
}

int gemm_mp_conversion_bytes(gemm_mp_ctx *c, size_t *bytes)
{
    if (!c || !bytes) return GEMM_MP_EINVAL;
    if (!all_maps(c)) return GEMM_MP_ESTATE;
    if (!c->sched_current) build_schedule(c);
    *bytes = (size_t)c->conv_bytes;
    return GEMM_MP_OK;
}

int gemm_mp_convert_tiles(gemm_mp_ctx *c, void *workspace, size_t bytes, gemm_mp_stream stream)
{
    if (!c) return GEMM_MP_EINVAL;
    Matrix &A = c->mat[0], &B = c->mat[1];
    if (!all_maps(c) || !A.packed || !B.packed) return GEMM_MP_ESTATE;
    size_t need = 0;
    int rc;
    if ((rc = gemm_mp_conversion_bytes(c, &need))) return rc;
    if (need > 0 && (!workspace || ((uintptr_t)workspace & 255) || bytes < need)) return GEMM_MP_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    if ((rc = ensure_tables(c, A, s)) || (rc = ensure_tables(c, B, s))) return rc;
    // jobs and address tables
    std::vector<ConvertJob> jobs;
    std::vector<uint64_t> addr[2];
    uint32_t max_n16 = 0;
    for (int w = 0; w < 2; ++w) {
        const Matrix &m = c->mat[w];
        addr[w].assign(c->conv_off[w].size(), 0);
        for (size_t k = 0; k < c->conv_off[w].size(); ++k) {
            if (c->conv_off[w][k] == kNoCopy) continue;
            const size_t tile = k / kConvSlots;
            const int q = (int)(k % kConvSlots);
            ConvertJob j;
            j.src = (uint64_t)(uintptr_t)((char *)m.storage + m.offset[tile]);
            j.dst = (uint64_t)(uintptr_t)((char *)workspace + c->conv_off[w][k]);
            j.tile = (uint32_t)tile;
            j.p = (uint8_t)m.map[tile];
            j.q = (uint8_t)q;
            j.which = (uint8_t)w;
            j.pad = 0;
            j.n16 = (uint32_t)(((uint64_t)c->nb * c->nb * elem_bytes(q)) / 16);
            j.nb = (uint32_t)c->nb;
            max_n16 = std::max(max_n16, j.n16);
            addr[w][k] = j.dst;
            jobs.push_back(j);
        }
    }
    // the tables may be in use by an earlier run on another stream
    if (c->d_conv[0]) { (void)hipStreamSynchronize(c->mat[2].last_stream); c->n_syncs += 1; }
    (void)hipFree(c->d_conv[0]); (void)hipFree(c->d_conv[1]); (void)hipFree(c->d_jobs);
    c->d_conv[0] = c->d_conv[1] = nullptr; c->d_jobs = nullptr;
    for (int w = 0; w < 2; ++w) {
        if ((rc = dev_alloc(c, &c->d_conv[w], addr[w].size()))) return rc;
        HIP_TRY(hipMemcpy(c->d_conv[w], addr[w].data(), addr[w].size() * sizeof(uint64_t), hipMemcpyHostToDevice));
    }
    if (!jobs.empty()) {
        if ((rc = dev_alloc(c, &c->d_jobs, jobs.size()))) return rc;
        HIP_TRY(hipMemcpy(c->d_jobs, jobs.data(), jobs.size() * sizeof(ConvertJob), hipMemcpyHostToDevice));
        HIP_TRY(launch_convert(c->d_jobs, (int)jobs.size(), max_n16, A.d_exp, B.d_exp, s));
    }
    A.last_stream = B.last_stream = s;
    c->conv_active = true;
    return GEMM_MP_OK;
}

int gemm_mp_clear_conversion(gemm_mp_ctx *c)
{
    if (!c) return GEMM_MP_EINVAL;
    c->conv_active = false;
    return GEMM_MP_OK;
}

int gemm_mp_tile_info(gemm_mp_ctx *c, char which, int32_t I, int32_t J, size_t *offset, int *prec, int *scale_exp)
{
    const int w = which_index(which);
    if (!c || w < 0) return GEMM_MP_EINVAL;
    Matrix &m = c->mat[w];
    if (!m.has_map) return GEMM_MP_ESTATE;
    if (I < 0 || I >= m.rows_t || J < 0 || J >= m.cols_t) return GEMM_MP_EINVAL;
    const int t = I * m.cols_t + J;
    int e = 0;
    if (scale_exp) {
        if (m.map[t] == GEMM_MP_FP16 || m.map[t] == GEMM_MP_FP8_E4M3) {
            if (!m.exps_valid) return GEMM_MP_ESTATE;
            if (int rc = host_wait(c, m.last_stream)) return rc;
            HIP_TRY(hipMemcpy(&e, m.d_exp + t, sizeof(int), hipMemcpyDeviceToHost));
        }
    }
    if (offset) *offset = (size_t)m.offset[t];
    if (prec) *prec = m.map[t];
    if (scale_exp) *scale_exp = e;
    return GEMM_MP_OK;
}

int gemm_mp_get_stats(gemm_mp_ctx *c, gemm_mp_stats *out)
{
    if (!c || !out) return GEMM_MP_EINVAL;
    if (!all_maps(c)) return GEMM_MP_ESTATE;
    if (!c->sched_current) build_schedule(c);
    *out = c->stats;
    out->converted_tiles = c->conv_active ? c->conv_tiles : 0;
    out->converted_bytes = c->conv_active ? c->conv_bytes : 0;
    return GEMM_MP_OK;
}

int gemm_mp_product_precision(int pA, int pB, int pC, int policy)
{
    if (pA < 0 || pA > 6 || pB < 0 || pB > 6 || pC < 0 || pC > 6) return -1;
    if (policy != GEMM_MP_POLICY_OPERAND && policy != GEMM_MP_POLICY_C_TILE) return -1;
    return product_precision(pA, pB, pC, policy);
}

const char *gemm_mp_strerror(int status)
{
    switch (status) {
    case GEMM_MP_OK: return "success";
    case GEMM_MP_EINVAL: return "invalid argument";
    case GEMM_MP_ESTATE: return "call order: a map, a buffer or packed data is missing";
    case GEMM_MP_ENOMEM: return "out of memory for a table";
    case GEMM_MP_EUNSUPPORTED: return "not supported by this build";
    case GEMM_MP_EHIP: return "HIP runtime error";
    case GEMM_MP_ETOOBIG: return "more tile products than the static scratch of gemm_mp_run_static holds";
    default: return "unknown status";
    }
}

}  // extern "C"
