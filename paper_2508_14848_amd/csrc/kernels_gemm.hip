// Host-side launch code of the GEMM step and its two small helper kernels: the product table
// (one record per tile product, gathered before every run) and the sender-side conversion of whole
// tiles.  The owner-workgroup kernels themselves are templates in gemm_owner_kernel.h (128 x 128
// regions) and gemm_region_kernel.h (256 x 256 regions), one instance per gemm_*.hip file.
#include "gemm_owner_kernel.h"

namespace gmp {

// One thread per task (C tile, L): gather what the owner workgroups need into one record.  With
// sender-side conversion a tile whose stored precision differs from the task's has a copy in
// that precision: the record then points there and carries the copy's precision (and, for
// FP64 / FP32 copies, exponent 0: the scale is already applied).
__global__ void product_table_kernel(PackedView A, PackedView B, const uint8_t *__restrict__ q, int MT, int NT, int KT,
                                     const uint64_t *__restrict__ convA, const uint64_t *__restrict__ convB,
                                     ProductDesc *__restrict__ out)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (int64_t)MT * NT * KT) return;
    const int L = (int)(idx % KT);
    const int tileC = (int)(idx / KT);
    const int I = tileC / NT, J = tileC % NT;
    const int64_t ta = (int64_t)I * KT + L, tb = (int64_t)L * NT + J;
    const uint32_t qq = q[idx];
    ProductDesc d;
    uint32_t pa = A.prec[ta], pb = B.prec[tb];
    d.a_ptr = (uint64_t)(uintptr_t)(A.storage + A.offset[ta]);
    d.b_ptr = (uint64_t)(uintptr_t)(B.storage + B.offset[tb]);
    d.ea = A.exp[ta];
    d.eb = B.exp[tb];
    if (convA && pa != qq && convA[ta * kConvSlots + qq]) {
        d.a_ptr = convA[ta * kConvSlots + qq];
        pa = qq;
        if (qq <= (uint32_t)Q32) d.ea = 0;
    }
    if (convB && pb != qq && convB[tb * kConvSlots + qq]) {
        d.b_ptr = convB[tb * kConvSlots + qq];
        pb = qq;
        if (qq <= (uint32_t)Q32) d.eb = 0;
    }
    // BF16 (code 4) has FP16's element size: the kernels see it as FP16 with a flag
    const uint32_t flags = (pa == GEMM_MP_BF16 ? 1u : 0u) | (pb == GEMM_MP_BF16 ? 2u : 0u) | (qq == GEMM_MP_BF16 ? 4u : 0u);
    const uint32_t ia = pa == GEMM_MP_BF16 ? (uint32_t)Q16 : pa, ib = pb == GEMM_MP_BF16 ? (uint32_t)Q16 : pb;
    const uint32_t iq = qq == GEMM_MP_BF16 ? (uint32_t)Q16 : qq;
    d.codes = ia | (ib << 8) | (iq << 16) | (flags << 24);
    d.pad = 0;
    out[idx] = d;
}

// Sender-side conversion of whole tiles: one thread per 16-byte segment of the result, using
// the very conversion the owner workgroups apply on the fly (convert<Q>), so a converted copy
// holds bit for bit what the receiver-side path would have put into LDS.
__global__ __launch_bounds__(256) void convert_tiles_kernel(const ConvertJob *__restrict__ jobs, const int32_t *__restrict__ expA,
                                                            const int32_t *__restrict__ expB, uint32_t per_job)
{
    // a one-dimensional grid: per_job workgroups for every job
    const ConvertJob job = jobs[blockIdx.x / per_job];
    const uint32_t seg = (blockIdx.x % per_job) * 256u + threadIdx.x;
    if (seg >= job.n16) return;
    const int p = job.p, q = job.q;
    if (p == GEMM_MP_MXFP4) {
        // MXFP4 tile to FP32 / FP64: e2m1 element times the scale of its block of 32 (exact)
        const uint8_t *sb = (const uint8_t *)(uintptr_t)job.src;
        const uint64_t elems = (uint64_t)job.n16 * (q == Q32 ? 4u : 2u);         // nb * nb
        const uint64_t idx = (uint64_t)seg * (q == Q32 ? 4u : 2u);                // first element of this segment: even
        const int sc = (int)sb[elems / 2 + (idx >> 5)] - 127;
        const uint32_t w = *(const uint16_t *)(sb + idx / 2 - ((idx / 2) & 1)) >> (8 * (int)((idx / 2) & 1));
        float v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int code = (int)(w >> (4 * k)) & 15, ef = (code >> 1) & 3, mf = code & 1;
            const float mag = ef ? ldexpf(1.0f + 0.5f * mf, ef - 1) : 0.5f * mf;
            v[k] = ldexpf((code & 8) ? -mag : mag, sc);
        }
        u32x4 o;
        if (q == Q32) o = u32x4{__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])};
        else {
            const u32x2 a = dbits((double)v[0]), b = dbits((double)v[1]);
            o = u32x4{a.x, a.y, b.x, b.y};
        }
        *(u32x4 *)((char *)(uintptr_t)job.dst + (uint64_t)seg * 16) = o;
        return;
    }
    if (p == GEMM_MP_MXFP6) {
        // MXFP6 tile to FP32 / FP64: e2m3 element times the scale of its block of 32 (exact); four
        // six-bit codes fill three bytes
        const uint8_t *sb = (const uint8_t *)(uintptr_t)job.src;
        const uint64_t elems = (uint64_t)job.n16 * (q == Q32 ? 4u : 2u);         // nb * nb
        const uint64_t idx = (uint64_t)seg * (q == Q32 ? 4u : 2u);                // first element of this segment: even
        const int sc = (int)sb[elems / 4 * 3 + (idx >> 5)] - 127;
        const int nb = (int)job.nb;
        const uint8_t *b3 = sb + fp6_group_offset(nb, (int)(idx / (uint64_t)nb), (int)(idx % (uint64_t)nb) & ~3);
        const uint32_t w = (b3[0] | ((uint32_t)b3[1] << 8) | ((uint32_t)b3[2] << 16)) >> (6 * (int)(idx & 3));
        float v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = ldexpf(fp6_value((w >> (6 * k)) & 63u), sc);
        u32x4 o;
        if (q == Q32) o = u32x4{__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])};
        else {
            const u32x2 a = dbits((double)v[0]), b = dbits((double)v[1]);
            o = u32x4{a.x, a.y, b.x, b.y};
        }
        *(u32x4 *)((char *)(uintptr_t)job.dst + (uint64_t)seg * 16) = o;
        return;
    }
    if (p == GEMM_MP_MXFP8) {
        // MXFP8 tile to FP32 / FP64: element times the scale of its block of 32 (exact)
        const uint8_t *sb = (const uint8_t *)(uintptr_t)job.src;
        const uint64_t elems = (uint64_t)job.n16 * (q == Q32 ? 4u : 2u);         // nb * nb; the scale bytes follow them
        u32x4 o;
        if (q == Q32) {
            const uint64_t idx = (uint64_t)seg * 4;
            const int w = (int)*(const uint32_t *)(sb + idx);
            const int sc = (int)sb[elems + (idx >> 5)] - 127;
            o = u32x4{__float_as_uint(ldexpf(__builtin_amdgcn_cvt_f32_fp8(w, 0), sc)), __float_as_uint(ldexpf(__builtin_amdgcn_cvt_f32_fp8(w, 1), sc)),
                      __float_as_uint(ldexpf(__builtin_amdgcn_cvt_f32_fp8(w, 2), sc)), __float_as_uint(ldexpf(__builtin_amdgcn_cvt_f32_fp8(w, 3), sc))};
        } else {
            const uint64_t idx = (uint64_t)seg * 2;
            const int w = (int)*(const uint16_t *)(sb + idx);
            const int sc = (int)sb[elems + (idx >> 5)] - 127;
            const u32x2 a = dbits(ldexp((double)__builtin_amdgcn_cvt_f32_fp8(w, 0), sc)), b = dbits(ldexp((double)__builtin_amdgcn_cvt_f32_fp8(w, 1), sc));
            o = u32x4{a.x, a.y, b.x, b.y};
        }
        *(u32x4 *)((char *)(uintptr_t)job.dst + (uint64_t)seg * 16) = o;
        return;
    }
    if (p == GEMM_MP_BF16 || q == GEMM_MP_BF16) {
        // BF16 tile to FP32 / FP64 (a shift: exact), or FP8 tile to BF16 keeping its scale (exact:
        // every e4m3 number is a BF16 number).  No other pair occurs: FP16 and BF16 meet in FP32.
        const char *sb = (const char *)(uintptr_t)job.src;
        u32x4 o;
        if (q == GEMM_MP_BF16) {
            const u32x2 w = *(const u32x2 *)(sb + (uint64_t)seg * 8);
            const int w0 = (int)w.x, w1 = (int)w.y;
            o.x = (__float_as_uint(__builtin_amdgcn_cvt_f32_fp8(w0, 0)) >> 16) | (__float_as_uint(__builtin_amdgcn_cvt_f32_fp8(w0, 1)) & 0xffff0000u);
            o.y = (__float_as_uint(__builtin_amdgcn_cvt_f32_fp8(w0, 2)) >> 16) | (__float_as_uint(__builtin_amdgcn_cvt_f32_fp8(w0, 3)) & 0xffff0000u);
            o.z = (__float_as_uint(__builtin_amdgcn_cvt_f32_fp8(w1, 0)) >> 16) | (__float_as_uint(__builtin_amdgcn_cvt_f32_fp8(w1, 1)) & 0xffff0000u);
            o.w = (__float_as_uint(__builtin_amdgcn_cvt_f32_fp8(w1, 2)) >> 16) | (__float_as_uint(__builtin_amdgcn_cvt_f32_fp8(w1, 3)) & 0xffff0000u);
        } else if (q == Q32) {
            const u32x2 w = *(const u32x2 *)(sb + (uint64_t)seg * 8);
            o = u32x4{w.x << 16, w.x & 0xffff0000u, w.y << 16, w.y & 0xffff0000u};
        } else {
            const uint32_t w = *(const uint32_t *)(sb + (uint64_t)seg * 4);
            const u32x2 a = dbits((double)__uint_as_float(w << 16)), b = dbits((double)__uint_as_float(w & 0xffff0000u));
            o = u32x4{a.x, a.y, b.x, b.y};
        }
        *(u32x4 *)((char *)(uintptr_t)job.dst + (uint64_t)seg * 16) = o;
        return;
    }
    const int e = (job.which == 0 ? expA : expB)[job.tile];
    const uint64_t src_byte = ((uint64_t)seg * (uint64_t)(2u << q)) << (3 - p);   // first source byte of this segment
    const char *src = (const char *)(uintptr_t)job.src + (src_byte & ~(uint64_t)15);
    Raw r;
    r.lo = *(const u32x4 *)src;
    r.hi = (q == Q32 && p == Q64) ? *(const u32x4 *)(src + 16) : r.lo;
    const int sub = (int)(src_byte & 15);
    u32x4 out;
    switch (q) {
    case Q64: out = convert<Q64>(r, p, e, sub); break;
    case Q32: out = convert<Q32>(r, p, e, sub); break;
    default:  out = convert<Q16>(r, p, e, sub); break;
    }
    *(u32x4 *)((char *)(uintptr_t)job.dst + (uint64_t)seg * 16) = out;
}

hipError_t launch_convert(const ConvertJob *jobs_dev, int njobs, uint32_t max_n16, const int32_t *expA, const int32_t *expB,
                          hipStream_t s)
{
    if (njobs <= 0) return hipSuccess;
    const uint32_t per_job = (max_n16 + 255u) / 256u;
    if ((int64_t)per_job * njobs > 0x7fffffff) return hipErrorInvalidValue;
    convert_tiles_kernel<<<dim3((unsigned)((int64_t)per_job * njobs)), dim3(256), 0, s>>>(jobs_dev, expA, expB, per_job);
    return hipGetLastError();
}

hipError_t gemm_kernel_setup()
{
    hipError_t (*const setups[13])() = {setup_owner_d_low, setup_owner_d, setup_owner_d_mixed, setup_owner_d_bf, setup_owner_f, setup_owner_f_mixed,
                                        setup_owner_f_bf, setup_region_fp8, setup_region_mxfp8, setup_region_mxfp4, setup_region_fp16,
                                        setup_region_bf16, setup_region_mxfp6};
    for (auto f : setups) {
        const hipError_t e = f();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// The product table, then one launch per kind of C tile: the owner regions of FP64 C tiles, those
// of FP32 C tiles, and the large regions of FP32 C tiles made of FP8 / MXFP8 / MXFP4 / FP16 / BF16 / MXFP6
// products only.
// The kinds touch disjoint C tiles and only read A, B and the tables, so they may run side by side:
// with `lanes` the first kind stays on the caller's stream and every further one goes to a side
// stream of its own, forked off behind the product table and joined again before the call
// returns to the caller's stream, so that workgroups of one kind fill the compute units the tail of
// another leaves idle.  Which workgroup computes what does not change: C is bit for bit the same.
hipError_t launch_gemm(const GemmArgs &a, hipStream_t s, const LaunchLanes *lanes)
{
    const int64_t tasks = (int64_t)a.MT * a.NT * a.KT;
    product_table_kernel<<<dim3((unsigned)((tasks + 255) / 256)), dim3(256), 0, s>>>(a.A, a.B, a.q, a.MT, a.NT, a.KT, a.convA, a.convB, a.prod);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    struct Kind {
        hipError_t (*launch)(const GemmArgs &, const WorkItem *, int, hipStream_t);
        const WorkItem *items;
        int n;
    };
    // BF16 tiles among the operands: the instances that know the BF16 matrix instruction; FP16 /
    // BF16 products with an FP8 operand: the instances whose DMA ring takes them; FP64 C tiles
    // without an FP64 product: the instance without the FP64 product loop
    const Kind all[8] = {
        {a.bf16 ? launch_owner_d_bf : a.mixed64 ? launch_owner_d_mixed : a.low64 ? launch_owner_d_low : launch_owner_d, a.items64, a.n_items64},
        {a.bf16 ? launch_owner_f_bf : a.mixed32 ? launch_owner_f_mixed : launch_owner_f, a.items32, a.n_items32},
        {launch_region_fp8, a.items8, a.n_items8},
        {launch_region_mxfp8, a.items_mx, a.n_items_mx},
        {launch_region_mxfp4, a.items_mx4, a.n_items_mx4},
        {launch_region_fp16, a.items_h, a.n_items_h},
        {launch_region_bf16, a.items_bf, a.n_items_bf},
        {launch_region_mxfp6, a.items_mx6, a.n_items_mx6}};
    Kind kinds[8];
    int n = 0;
    for (const Kind &k : all)
        if (k.n > 0) kinds[n++] = k;
    if (n <= 1 || !lanes) {
        for (int i = 0; i < n; ++i)
            if ((e = kinds[i].launch(a, kinds[i].items, kinds[i].n, s)) != hipSuccess) return e;
        return hipSuccess;
    }
    if ((e = hipEventRecord(lanes->fork, s)) != hipSuccess) return e;
    if ((e = kinds[0].launch(a, kinds[0].items, kinds[0].n, s)) != hipSuccess) return e;
    for (int i = 1; i < n; ++i) {
        hipStream_t side = lanes->side[(i - 1) % 4];
        if ((e = hipStreamWaitEvent(side, lanes->fork, 0)) != hipSuccess) return e;
        if ((e = kinds[i].launch(a, kinds[i].items, kinds[i].n, side)) != hipSuccess) return e;
    }
    for (int i = 1; i < n && i <= 4; ++i) {          // every side stream joins once, behind its last launch
        if ((e = hipEventRecord(lanes->join[i - 1], lanes->side[i - 1])) != hipSuccess) return e;
        if ((e = hipStreamWaitEvent(s, lanes->join[i - 1], 0)) != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace gmp
