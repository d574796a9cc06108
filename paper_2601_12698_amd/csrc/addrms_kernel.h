// Device-side template of the fused residual-add + RMSNorm kernel for gfx950.
//
// This is the "parameterizable template" of the paper's Level 2 (Algorithm 1,
// Templatize; Section 3.3 lists the knob families: thread-level granularity,
// loop scheduling/unrolling, vectorisation/alignment, organisation of shared
// memory and registers).  The knobs are
//
//   VEC   elements per thread per chunk (one vector load of x, one of residual)
//   CPT   chunks per thread = ceil(N / (VEC * threads_per_row)); the whole row
//         slice lives in registers between the two passes (register row cache)
//   UNR   chunks whose loads are in flight before the first one is consumed
//   threads_per_row, rows_per_wg : launch shape (blockDim.x, blockDim.y)
//   reduce  : wave64 cross-lane (DPP) sums + one LDS hop across waves, or an
//             LDS-staged tree
//   NT    non-temporal (streaming) cache policy on the x and residual loads
//         and stores; the weight vector always uses the default policy
//   DEFER residual stored after the row reduction, all of its chunks first and
//         then those of y, instead of chunk by chunk as the sums are formed: a
//         workgroup then reads in one phase and writes in one phase, and no load
//         is ever issued behind a store whose acknowledgement the wave would have
//         to wait for (loads and stores share one in-order counter on this target)
//   flags   : XCD-contiguous mapping of workgroups to rows; persistent grid
//             (set by the host through the grid size: fewer workgroups than
//             row blocks makes each workgroup loop with a prefetch)
//
// VEC, CPT, UNR, NT and DEFER are compile-time; the rest are launch-time and
// uniform over the workgroup.
//
// Arithmetic per row (what every instantiation must reproduce bit for bit):
//   h = f32(x) + f32(r)                       one fp32 add
//   residual <- RNE(h -> residual dtype)      in place
//   ss = sum h^2  accumulated in fp64 (each h^2 is exact in fp64), any order
//   rstd = fp32( rsqrt(ss * (1/N) + eps) )    fp64, refined to fp64 accuracy
//   x <- RNE((h * rstd) * f32(w) -> x dtype)  two fp32 multiplies, in place
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace addrms {

enum : int { DT_BF16 = 0, DT_FP16 = 1, DT_FP16_RES32 = 2, DT_FP32 = 3 };
enum : int { RED_WAVE = 0, RED_LDS = 1 };
enum : uint32_t { FLAG_XCD_CONTIG = 1u, FLAG_NONTEMPORAL = 2u, FLAG_PERSISTENT = 4u, FLAG_TWO_PASS = 8u,
                  FLAG_LDS_CACHE = 16u, FLAG_DEFER_STORE = 32u, FLAG_ALIGNED_SPAN = 64u };

template <int DT> struct dt_traits;
template <> struct dt_traits<DT_BF16>       { static constexpr int XB = 2, RB = 2; static constexpr bool BF = true;  };
template <> struct dt_traits<DT_FP16>       { static constexpr int XB = 2, RB = 2; static constexpr bool BF = false; };
template <> struct dt_traits<DT_FP16_RES32> { static constexpr int XB = 2, RB = 4; static constexpr bool BF = false; };
template <> struct dt_traits<DT_FP32>       { static constexpr int XB = 4, RB = 4; static constexpr bool BF = false; };

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// Raw register image of one vector access of BYTES bytes (2..32).
template <int BYTES> struct raw_t { uint32_t d[(BYTES + 3) / 4]; };

template <bool NT, typename T>
__device__ __forceinline__ T ld_as(const char* p)
{
    if constexpr (NT) return __builtin_nontemporal_load(reinterpret_cast<const T*>(p));
    else return *reinterpret_cast<const T*>(p);
}
template <bool NT, typename T>
__device__ __forceinline__ void st_as(char* p, T v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, reinterpret_cast<T*>(p));
    else *reinterpret_cast<T*>(p) = v;
}

template <int BYTES, bool NT = false>
__device__ __forceinline__ void ld_raw(const char* p, raw_t<BYTES>& v)
{
    if constexpr (BYTES == 2) {
        v.d[0] = ld_as<NT, uint16_t>(p);
    } else if constexpr (BYTES == 4) {
        v.d[0] = ld_as<NT, uint32_t>(p);
    } else if constexpr (BYTES == 8) {
        u32x2 t = ld_as<NT, u32x2>(p);
        v.d[0] = t.x; v.d[1] = t.y;
    } else if constexpr (BYTES == 16) {
        u32x4 t = ld_as<NT, u32x4>(p);
        v.d[0] = t.x; v.d[1] = t.y; v.d[2] = t.z; v.d[3] = t.w;
    } else {
        static_assert(BYTES == 32, "vector access must be 2, 4, 8, 16 or 32 bytes");
        u32x4 a = ld_as<NT, u32x4>(p);
        u32x4 b = ld_as<NT, u32x4>(p + 16);
        v.d[0] = a.x; v.d[1] = a.y; v.d[2] = a.z; v.d[3] = a.w;
        v.d[4] = b.x; v.d[5] = b.y; v.d[6] = b.z; v.d[7] = b.w;
    }
}

template <int BYTES, bool NT = false>
__device__ __forceinline__ void st_raw(char* p, const raw_t<BYTES>& v)
{
    if constexpr (BYTES == 2) {
        st_as<NT, uint16_t>(p, static_cast<uint16_t>(v.d[0]));
    } else if constexpr (BYTES == 4) {
        st_as<NT, uint32_t>(p, v.d[0]);
    } else if constexpr (BYTES == 8) {
        u32x2 t = {v.d[0], v.d[1]};
        st_as<NT, u32x2>(p, t);
    } else if constexpr (BYTES == 16) {
        u32x4 t = {v.d[0], v.d[1], v.d[2], v.d[3]};
        st_as<NT, u32x4>(p, t);
    } else {
        static_assert(BYTES == 32, "vector access must be 2, 4, 8, 16 or 32 bytes");
        u32x4 a = {v.d[0], v.d[1], v.d[2], v.d[3]};
        u32x4 b = {v.d[4], v.d[5], v.d[6], v.d[7]};
        st_as<NT, u32x4>(p, a);
        st_as<NT, u32x4>(p + 16, b);
    }
}

// Element e of a raw vector of ES-byte elements, widened to fp32 (exact).
template <int ES, bool BF, int BYTES>
__device__ __forceinline__ float get_elem(const raw_t<BYTES>& v, int e)
{
    if constexpr (ES == 4) {
        return __uint_as_float(v.d[e]);
    } else {
        const uint32_t dw = v.d[e >> 1];
        if constexpr (BF) {
            return __uint_as_float((e & 1) ? (dw & 0xffff0000u) : (dw << 16));
        } else {
            f16x2 hh = __builtin_bit_cast(f16x2, dw);
            return (e & 1) ? static_cast<float>(hh.y) : static_cast<float>(hh.x);
        }
    }
}

// Two fp32 values rounded to nearest-even into one dword of 16-bit storage.
// The empty asm pins both values in registers as finished fp32 results: without
// it the compiler may fold the preceding fp32 multiply and this conversion into
// one mixed-precision multiply that rounds once, which differs from rounding
// the fp32 product first whenever that product is an exact tie of the format.
template <bool BF>
__device__ __forceinline__ uint32_t pack2(float lo, float hi)
{
    asm volatile("" : "+v"(lo), "+v"(hi));
    f32x2 f = {lo, hi};
    if constexpr (BF) {
        bf16x2 b = __builtin_convertvector(f, bf16x2);
        return __builtin_bit_cast(uint32_t, b);
    } else {
        f16x2 b = __builtin_convertvector(f, f16x2);
        return __builtin_bit_cast(uint32_t, b);
    }
}

// VEC fp32 values -> raw vector of ES-byte elements.
template <int ES, bool BF, int VEC>
__device__ __forceinline__ void pack_vec(const float (&f)[VEC], raw_t<ES * VEC>& out)
{
    if constexpr (ES == 4) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) out.d[e] = __float_as_uint(f[e]);
    } else if constexpr (VEC == 1) {
        out.d[0] = pack2<BF>(f[0], 0.0f) & 0xffffu;
    } else {
#pragma unroll
        for (int e = 0; e < VEC; e += 2) out.d[e >> 1] = pack2<BF>(f[e], f[e + 1]);
    }
}

// ---- cross-lane movement of one dword ------------------------------------
// xor-butterfly partner fetch.  Steps 1, 2 use DPP quad permutes; 4 and 8 use
// the DPP half-row and row mirrors (valid as butterfly steps because the
// lanes being mirrored already hold equal sub-sums); 16 uses the LDS crossbar
// swizzle; 32 uses a wave-wide bpermute.
template <int STEP>
__device__ __forceinline__ uint32_t lane_partner(uint32_t v)
{
    if constexpr (STEP == 1) {
        return __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, true);   // quad_perm [1,0,3,2]
    } else if constexpr (STEP == 2) {
        return __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, true);   // quad_perm [2,3,0,1]
    } else if constexpr (STEP == 4) {
        return __builtin_amdgcn_update_dpp(0, v, 0x141, 0xF, 0xF, true);  // row_half_mirror
    } else if constexpr (STEP == 8) {
        return __builtin_amdgcn_update_dpp(0, v, 0x140, 0xF, 0xF, true);  // row_mirror
    } else if constexpr (STEP == 16) {
        return __builtin_amdgcn_ds_swizzle(v, 0x401F);                    // lane ^ 16 within 32
    } else {
        static_assert(STEP == 32, "butterfly step");
        const uint32_t self = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
        return __builtin_amdgcn_ds_bpermute(static_cast<int>((self ^ 32u) << 2), v);
    }
}

template <int STEP>
__device__ __forceinline__ double butterfly_add(double v)
{
    const uint64_t bits = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = lane_partner<STEP>(static_cast<uint32_t>(bits));
    const uint32_t hi = lane_partner<STEP>(static_cast<uint32_t>(bits >> 32));
    const double other = __builtin_bit_cast(double, (static_cast<uint64_t>(hi) << 32) | lo);
    return v + other;       // a+b on one side, b+a on the other: identical bits
}

// Sum over aligned groups of `width` lanes (8, 16 or 32: rows narrower than a wave;
// 64 works too); every lane of a group ends with the same bits.
__device__ __forceinline__ double wave_group_sum(double v, uint32_t width)
{
    v = butterfly_add<1>(v);
    v = butterfly_add<2>(v);
    v = butterfly_add<4>(v);
    if (width >= 16) v = butterfly_add<8>(v);
    if (width >= 32) v = butterfly_add<16>(v);
    if (width >= 64) v = butterfly_add<32>(v);
    return v;
}

// ---- sums that end in one lane and are broadcast from there ---------------------------------
// One dword-pair DPP move; lanes the move does not reach (outside the row for a shift, masked rows or banks) read 0.0.
template <int CTRL, int ROW_MASK, int BANK_MASK>
__device__ __forceinline__ double dpp_or_zero(double v)
{
    const uint64_t bits = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = __builtin_amdgcn_update_dpp(0u, static_cast<uint32_t>(bits), CTRL, ROW_MASK, BANK_MASK, false);
    const uint32_t hi = __builtin_amdgcn_update_dpp(0u, static_cast<uint32_t>(bits >> 32), CTRL, ROW_MASK, BANK_MASK, false);
    return __builtin_bit_cast(double, (static_cast<uint64_t>(hi) << 32) | lo);
}
// Inclusive scan over each DPP row of 16 lanes (row_shr 1, 2, 4, 8 with zero fill): lane 15 of a row ends with
// the row's sum.
__device__ __forceinline__ double row16_scan(double v)
{
    v += dpp_or_zero<0x111, 0xF, 0xF>(v);
    v += dpp_or_zero<0x112, 0xF, 0xF>(v);
    v += dpp_or_zero<0x114, 0xF, 0xF>(v);
    v += dpp_or_zero<0x118, 0xF, 0xF>(v);
    return v;
}
__device__ __forceinline__ double read_lane(double v, int lane)
{
    const uint64_t bits = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(static_cast<uint32_t>(bits)), lane));
    const uint32_t hi = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(static_cast<uint32_t>(bits >> 32)), lane));
    return __builtin_bit_cast(double, (static_cast<uint64_t>(hi) << 32) | lo);
}
// Sum over all 64 lanes, the same bits in every lane: four scan steps inside the DPP rows, the row sums carried
// into the following rows by the two row broadcasts (lane 15 of rows 0 and 2 into rows 1 and 3, then lane 31 into
// rows 2 and 3), the total read from lane 63.  Vector ALU only: nothing goes through the LDS crossbar.
__device__ __forceinline__ double wave_total(double v)
{
    v = row16_scan(v);
    v += dpp_or_zero<0x142, 0xA, 0xF>(v);       // row_bcast:15
    v += dpp_or_zero<0x143, 0xC, 0xF>(v);       // row_bcast:31
    return read_lane(v, 63);
}

// Workgroup barrier that orders LDS traffic only.  The generic barrier also makes a wave wait until every global
// load and store it has issued is complete: a workgroup would wait for the acknowledgement of the stores it has
// just issued, and for loads it has issued ahead for its next row block, each time it reduces a row.  In these
// kernels threads exchange data through LDS alone (no thread reads global memory that another thread of the same
// launch wrote), so global traffic may stay in flight across the barrier.
__device__ __forceinline__ void wg_sync_lds()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Row sum of per-thread partials; result identical in all threads of the row.
// lds: RED_WAVE needs rows_per_wg * 16 doubles, RED_LDS needs one double per thread.
__device__ __forceinline__ double row_sum(double part, int reduce, uint32_t tpr, uint32_t lane, uint32_t ry,
                                          double* lds)
{
    if (reduce == RED_WAVE) {
        if (tpr < 64u) return wave_group_sum(part, tpr);
        const double wsum = wave_total(part);
        if (tpr == 64u) return wsum;
        const uint32_t nw = tpr >> 6;                 // 2..16 waves share the row
        double* slot = lds + ry * 16u;
        if ((lane & 63u) == 0u) slot[lane >> 6] = wsum;
        wg_sync_lds();
        // Every wave adds the nw wave sums the same way: one LDS read per lane, a scan over 16 lanes, lane 15
        // broadcast.  (A loop over the slots is a chain of dependent LDS reads: with 14 waves per row it cost
        // 3.6 % of the whole kernel's time.)
        const uint32_t k = lane & 15u;
        const double mine = k < nw ? slot[k] : 0.0;
        return read_lane(row16_scan(mine), 15);
    }
    double* buf = lds + ry * tpr;
    buf[lane] = part;
    wg_sync_lds();
    uint32_t cur = tpr;
    while (cur > 1u) {
        const uint32_t half = (cur + 1u) >> 1;
        if (lane + half < cur) buf[lane] += buf[lane + half];
        wg_sync_lds();
        cur = half;
    }
    return buf[0];
}

// fp32 rounding of 1/sqrt(d) for d > 0 in fp64: hardware estimate refined by
// two Newton steps, which leaves an error of a few fp64 ulps -- 2^29 times
// finer than the fp32 cell the result is rounded into.
__device__ __forceinline__ float rsqrt_to_f32(double d)
{
    double y = __builtin_amdgcn_rsq(d);
    if (d > 0.0 && d < __builtin_huge_val()) {
        const double hd = 0.5 * d;
        y = y * __builtin_fma(-hd * y, y, 1.5);
        y = y * __builtin_fma(-hd * y, y, 1.5);
    }
    return static_cast<float>(y);
}

// Workgroup b of nb -> position in row order such that the workgroups that
// land on one XCD (dispatch is round-robin over 8 XCDs) cover one contiguous
// range of rows.  Bijective for any nb.
__device__ __forceinline__ uint32_t xcd_contiguous(uint32_t b, uint32_t nb)
{
    const uint32_t xcd = b & 7u, idx = b >> 3;
    const uint32_t q = nb >> 3, rem = nb & 7u;
    return xcd * q + (xcd < rem ? xcd : rem) + idx;
}

// Per-workgroup-iteration addressing: base pointers are wave-uniform (SGPRs), the
// per-thread part fits 32 bits.
struct RowAddr {
    char* xbase;
    char* rbase;
    uint32_t rowoff;   // elements from the workgroup's first row to this thread's row
    uint32_t row_ok;   // 1 if this thread's row exists (the last workgroup may be ragged)
};

template <int XB, int RB>
__device__ __forceinline__ RowAddr row_addr(void* xp, void* rp, uint32_t blk, uint32_t rpw, uint32_t ry,
                                            int64_t M, int32_t N)
{
    RowAddr a;
    const int64_t row0 = static_cast<int64_t>(blk) * rpw;
    const int64_t left = M - row0;                          // rows available to this block (>= 1)
    a.row_ok = static_cast<int64_t>(ry) < left ? 1u : 0u;
    const uint32_t ryc = a.row_ok ? ry : static_cast<uint32_t>(left - 1);   // ghost threads re-read the last row
    a.xbase = static_cast<char*>(xp) + row0 * N * XB;
    a.rbase = static_cast<char*>(rp) + row0 * N * RB;
    a.rowoff = ryc * static_cast<uint32_t>(N);
    return a;
}

// Issues the loads of chunk group g (UNR chunks starting at chunk g) of one row.
template <int XB, int RB, int VEC, int CPT, int UNR, bool NT>
__device__ __forceinline__ void load_group(const char* xbase, const char* rbase, uint32_t rowoff, uint32_t col0,
                                           uint32_t stride, uint32_t nlast, int g,
                                           raw_t<XB * VEC> (&xv)[UNR], raw_t<RB * VEC> (&rv)[UNR])
{
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
        if (g + u < CPT) {
            const uint32_t col = col0 + static_cast<uint32_t>(g + u) * stride;
            const uint32_t colc = col < nlast ? col : nlast;      // clamp: tail lanes re-read valid data
            ld_raw<XB * VEC, NT>(xbase + static_cast<uint64_t>((rowoff + colc) * XB), xv[u]);
            ld_raw<RB * VEC, NT>(rbase + static_cast<uint64_t>((rowoff + colc) * RB), rv[u]);
        }
    }
}

// The grid has either one workgroup per block of rows_per_wg rows, or fewer
// (a persistent grid sized to what is resident on the chip): a workgroup then
// walks blocks blk, blk + gridDim.x, ... and issues the first loads of its
// next block before reducing the current one, so that it always has requests
// in flight.  Every workgroup leaves the loop after its last block; there is
// no waiting between workgroups.
template <int DT, int VEC, int CPT, int UNR, bool NT, bool DEFER>
__device__ __forceinline__ void addrms_body(void* __restrict__ xp, void* __restrict__ rp,
                                            const void* __restrict__ wp, float eps, double inv_n,
                                            int64_t M, int32_t N, uint32_t flags, int32_t reduce,
                                            uint32_t nblocks)
{
    using T = dt_traits<DT>;
    constexpr int XB = T::XB, RB = T::RB;
    constexpr bool BF = T::BF;
    extern __shared__ double lds[];

    const uint32_t tpr = blockDim.x, rpw = blockDim.y;
    const uint32_t lane = threadIdx.x, ry = threadIdx.y;
    uint32_t blk = blockIdx.x;
    if (flags & FLAG_XCD_CONTIG) blk = xcd_contiguous(blk, gridDim.x);

    const char* wbase = static_cast<const char*>(wp);
    const uint32_t col0 = lane * VEC;
    const uint32_t stride = tpr * VEC;
    const uint32_t nlast = static_cast<uint32_t>(N) - VEC;
    // LDS region of one reduction; consecutive iterations alternate between two regions
    const uint32_t lds_region = (reduce == RED_WAVE) ? rpw * 16u : rpw * tpr;

    raw_t<XB * VEC> xv[UNR];
    raw_t<RB * VEC> rv[UNR];
    RowAddr ra = row_addr<XB, RB>(xp, rp, blk, rpw, ry, M, N);
    load_group<XB, RB, VEC, CPT, UNR, NT>(ra.xbase, ra.rbase, ra.rowoff, col0, stride, nlast, 0, xv, rv);

    uint32_t parity = 0;
    const uint32_t col_first = col0;
    for (;;) {
        // Column offsets are recomputed in every iteration on purpose: hoisting them out of
        // the row loop would keep several registers per chunk alive across the whole loop.
        uint32_t col0 = col_first;
        asm volatile("" : "+v"(col0));
        float h[CPT][VEC];
        double acc = 0.0;
#pragma unroll
        for (int g = 0; g < CPT; g += UNR) {
            if (g > 0)    // group 0 was issued ahead (prologue or previous iteration)
                load_group<XB, RB, VEC, CPT, UNR, NT>(ra.xbase, ra.rbase, ra.rowoff, col0, stride, nlast, g, xv, rv);
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                if (g + u < CPT) {
                    const int c = g + u;
                    const uint32_t col = col0 + static_cast<uint32_t>(c) * stride;
#pragma unroll
                    for (int e = 0; e < VEC; ++e)
                        h[c][e] = get_elem<XB, BF>(xv[u], e) + get_elem<RB, BF && RB == 2>(rv[u], e);
                    if (ra.row_ok && col <= nlast) {
                        if constexpr (!DEFER) {
                            raw_t<RB * VEC> out;
                            pack_vec<RB, BF, VEC>(h[c], out);
                            st_raw<RB * VEC, NT>(ra.rbase + static_cast<uint64_t>((ra.rowoff + col) * RB), out);
                        }
#pragma unroll
                        for (int e = 0; e < VEC; ++e) {
                            const double hd = static_cast<double>(h[c][e]);
                            acc = __builtin_fma(hd, hd, acc);
                        }
                    }
                }
            }
            if (g + UNR < CPT) __builtin_amdgcn_sched_barrier(0);
        }

        const uint32_t next = blk + gridDim.x;
        const bool more = next < nblocks;         // uniform over the workgroup
        RowAddr rn = ra;
        if (more) {
            rn = row_addr<XB, RB>(xp, rp, next, rpw, ry, M, N);
            load_group<XB, RB, VEC, CPT, UNR, NT>(rn.xbase, rn.rbase, rn.rowoff, col0, stride, nlast, 0, xv, rv);
        }

        // Weights: tiny and L2/L1-resident after the first workgroups; issued before the
        // reduction so their latency hides behind it.
        raw_t<XB * VEC> wv[CPT];
#pragma unroll
        for (int c = 0; c < CPT; ++c) {
            const uint32_t col = col0 + static_cast<uint32_t>(c) * stride;
            const uint32_t colc = col < nlast ? col : nlast;
            ld_raw<XB * VEC>(wbase + static_cast<uint64_t>(colc * XB), wv[c]);
        }

        const double ss = row_sum(acc, reduce, tpr, lane, ry, lds + parity * lds_region);
        const float rstd = rsqrt_to_f32(__builtin_fma(ss, inv_n, static_cast<double>(eps)));

        if constexpr (DEFER) {      // the write phase: the whole residual row, then the whole y row
#pragma unroll
            for (int c = 0; c < CPT; ++c) {
                const uint32_t col = col0 + static_cast<uint32_t>(c) * stride;
                if (ra.row_ok && col <= nlast) {
                    raw_t<RB * VEC> out;
                    pack_vec<RB, BF, VEC>(h[c], out);
                    st_raw<RB * VEC, NT>(ra.rbase + static_cast<uint64_t>((ra.rowoff + col) * RB), out);
                }
            }
        }
#pragma unroll
        for (int c = 0; c < CPT; ++c) {
            const uint32_t col = col0 + static_cast<uint32_t>(c) * stride;
            float y[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const float t = h[c][e] * rstd;
                y[e] = t * get_elem<XB, BF>(wv[c], e);
            }
            if (ra.row_ok && col <= nlast) {
                raw_t<XB * VEC> out;
                pack_vec<XB, BF, VEC>(y, out);
                st_raw<XB * VEC, NT>(ra.xbase + static_cast<uint64_t>((ra.rowoff + col) * XB), out);
            }
        }
        if (!more) break;
        ra = rn;
        blk = next;
        parity ^= 1u;
    }
}

// Two-pass form for rows that do not fit the register row cache.  Pass 1 reads the
// row and accumulates the sum of squares; pass 2 reads it again, recomputes the same
// fp32 sums, and writes both outputs.  Nothing is written before the whole row has
// been summed, and every element is re-read and written by the lane that summed it,
// so the in-place update is safe.  Pass 1 loads with the default cache policy so that
// the second read of a row can be served from the L2 it was just pulled through;
// NT selects the streaming policy for the pass-2 loads (last use) and the stores.
// UNR chunks per stream are in flight per loop iteration.  The loop count is uniform
// over the workgroup; lanes past the end of the row are predicated off (N is a
// multiple of VEC, so a chunk is either wholly inside the row or wholly outside).
template <int DT, int VEC, int UNR, bool NT>
__device__ __forceinline__ void addrms_twopass_body(void* __restrict__ xp, void* __restrict__ rp,
                                                    const void* __restrict__ wp, float eps, double inv_n,
                                                    int64_t M, int32_t N, uint32_t flags, int32_t reduce,
                                                    uint32_t nblocks)
{
    using T = dt_traits<DT>;
    constexpr int XB = T::XB, RB = T::RB;
    constexpr bool BF = T::BF;
    extern __shared__ double lds[];
    (void)nblocks;

    const uint32_t tpr = blockDim.x, rpw = blockDim.y;
    const uint32_t lane = threadIdx.x, ry = threadIdx.y;
    uint32_t blk = blockIdx.x;
    if (flags & FLAG_XCD_CONTIG) blk = xcd_contiguous(blk, gridDim.x);

    const RowAddr ra = row_addr<XB, RB>(xp, rp, blk, rpw, ry, M, N);
    const char* wbase = static_cast<const char*>(wp);
    const uint32_t n = static_cast<uint32_t>(N);
    const uint32_t stride = tpr * VEC;
    const uint32_t span = stride * UNR;                        // elements of a row covered per iteration
    const uint32_t iters = (n + span - 1u) / span;
    const uint32_t col_first = lane * VEC;

    double acc = 0.0;
    for (uint32_t it = 0; it < iters; ++it) {
        raw_t<XB * VEC> xv[UNR];
        raw_t<RB * VEC> rv[UNR];
        const uint32_t col0 = col_first + it * span;
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const uint32_t col = col0 + static_cast<uint32_t>(u) * stride;
            if (col < n) {
                ld_raw<XB * VEC, false>(ra.xbase + static_cast<uint64_t>((ra.rowoff + col) * XB), xv[u]);
                ld_raw<RB * VEC, false>(ra.rbase + static_cast<uint64_t>((ra.rowoff + col) * RB), rv[u]);
            }
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const uint32_t col = col0 + static_cast<uint32_t>(u) * stride;
            if (ra.row_ok && col < n) {
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const float h = get_elem<XB, BF>(xv[u], e) + get_elem<RB, BF && RB == 2>(rv[u], e);
                    const double hd = static_cast<double>(h);
                    acc = __builtin_fma(hd, hd, acc);
                }
            }
        }
    }

    const double ss = row_sum(acc, reduce, tpr, lane, ry, lds);
    const float rstd = rsqrt_to_f32(__builtin_fma(ss, inv_n, static_cast<double>(eps)));

    // Pass 2 walks the row backwards: its end was read last in pass 1 and is the part most
    // likely to be still in the L2.
    for (uint32_t k = 0; k < iters; ++k) {
        const uint32_t it = iters - 1u - k;
        raw_t<XB * VEC> xv[UNR], wv[UNR];
        raw_t<RB * VEC> rv[UNR];
        const uint32_t col0 = col_first + it * span;
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const uint32_t col = col0 + static_cast<uint32_t>(u) * stride;
            if (col < n) {
                ld_raw<XB * VEC, NT>(ra.xbase + static_cast<uint64_t>((ra.rowoff + col) * XB), xv[u]);
                ld_raw<RB * VEC, NT>(ra.rbase + static_cast<uint64_t>((ra.rowoff + col) * RB), rv[u]);
                ld_raw<XB * VEC>(wbase + static_cast<uint64_t>(col * XB), wv[u]);
            }
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const uint32_t col = col0 + static_cast<uint32_t>(u) * stride;
            if (ra.row_ok && col < n) {
                float h[VEC], y[VEC];
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    h[e] = get_elem<XB, BF>(xv[u], e) + get_elem<RB, BF && RB == 2>(rv[u], e);
                    const float t = h[e] * rstd;
                    y[e] = t * get_elem<XB, BF>(wv[u], e);
                }
                raw_t<RB * VEC> rout;
                pack_vec<RB, BF, VEC>(h, rout);
                st_raw<RB * VEC, NT>(ra.rbase + static_cast<uint64_t>((ra.rowoff + col) * RB), rout);
                raw_t<XB * VEC> yout;
                pack_vec<XB, BF, VEC>(y, yout);
                st_raw<XB * VEC, NT>(ra.xbase + static_cast<uint64_t>((ra.rowoff + col) * XB), yout);
            }
        }
    }
}

// The one body of the forms whose row cache continues in LDS.  The first CPT chunks of a thread
// stay in registers (48 values: a 1024-thread workgroup leaves each lane 128 registers); the fp32
// sums of the next `lds_chunks` are parked in the thread's own slots of the workgroup's LDS
// allocation (laid out [row][chunk][lane][vec] behind the reduction scratch, so no other thread
// touches them) and read back once rstd is known.  LDS-continued cache: that covers the whole
// row, one pass.  Hybrid form (both long-row flags, rows beyond registers + LDS): only the
// remaining chunks are treated as in the two-pass form: summed in pass 1 without being written,
// re-read in pass 2 (backwards, so that what pass 1 pulled through the caches last is asked for
// first) to form both outputs.  The part of the row that is read twice shrinks from all of it to
// what does not fit on the chip.
// lds_chunks comes from the host, which sized the LDS allocation (it travels in the kernel
// argument the persistent forms use for the number of row blocks); fewer chunks than CPT +
// lds_chunks simply leave the tail of the register part idle (clamped loads, no stores).
template <int DT, int VEC, int CPT, int UNR, bool NT>
__device__ __forceinline__ void addrms_hybrid_body(void* __restrict__ xp, void* __restrict__ rp,
                                                   const void* __restrict__ wp, float eps, double inv_n,
                                                   int64_t M, int32_t N, uint32_t flags, int32_t reduce,
                                                   uint32_t lds_chunks)
{
    using T = dt_traits<DT>;
    constexpr int XB = T::XB, RB = T::RB;
    constexpr bool BF = T::BF;
    extern __shared__ double lds[];

    const uint32_t tpr = blockDim.x, rpw = blockDim.y;
    const uint32_t lane = threadIdx.x, ry = threadIdx.y;
    uint32_t blk = blockIdx.x;
    if (flags & FLAG_XCD_CONTIG) blk = xcd_contiguous(blk, gridDim.x);

    const RowAddr ra = row_addr<XB, RB>(xp, rp, blk, rpw, ry, M, N);
    const char* wbase = static_cast<const char*>(wp);
    const uint32_t n = static_cast<uint32_t>(N);
    const uint32_t stride = tpr * VEC;
    const uint32_t nlast = n - VEC;
    const uint32_t col0 = lane * VEC;
    const uint32_t need = (n + stride - 1u) / stride;                      // chunks per thread (host: need > CPT + lds_chunks)
    const uint32_t first_streamed = CPT + lds_chunks;
    const uint32_t red_doubles = (reduce == RED_WAVE) ? (tpr > 64u ? rpw * 16u : 0u) : rpw * tpr;
    float* cache = reinterpret_cast<float*>(lds + red_doubles) + (static_cast<size_t>(ry) * lds_chunks * tpr + lane) * VEC;
    const uint32_t cache_step = tpr * VEC;

    float h[CPT][VEC];
    double acc = 0.0;
    // ---- register part
#pragma unroll
    for (int g = 0; g < CPT; g += UNR) {
        raw_t<XB * VEC> xv[UNR];
        raw_t<RB * VEC> rv[UNR];
        load_group<XB, RB, VEC, CPT, UNR, NT>(ra.xbase, ra.rbase, ra.rowoff, col0, stride, nlast, g, xv, rv);
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            if (g + u < CPT) {
                const int c = g + u;
                const uint32_t col = col0 + static_cast<uint32_t>(c) * stride;
#pragma unroll
                for (int e = 0; e < VEC; ++e)
                    h[c][e] = get_elem<XB, BF>(xv[u], e) + get_elem<RB, BF && RB == 2>(rv[u], e);
                if (ra.row_ok && col <= nlast) {
                    raw_t<RB * VEC> out;
                    pack_vec<RB, BF, VEC>(h[c], out);
                    st_raw<RB * VEC, NT>(ra.rbase + static_cast<uint64_t>((ra.rowoff + col) * RB), out);
#pragma unroll
                    for (int e = 0; e < VEC; ++e) {
                        const double hd = static_cast<double>(h[c][e]);
                        acc = __builtin_fma(hd, hd, acc);
                    }
                }
            }
        }
        if (g + UNR < CPT) __builtin_amdgcn_sched_barrier(0);
    }
    // ---- LDS part
    for (uint32_t e0 = 0; e0 < lds_chunks; e0 += UNR) {
        raw_t<XB * VEC> xv[UNR];
        raw_t<RB * VEC> rv[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            if (e0 + u < lds_chunks) {
                const uint32_t col = col0 + (CPT + e0 + u) * stride;
                const uint32_t colc = col < nlast ? col : nlast;
                ld_raw<XB * VEC, NT>(ra.xbase + static_cast<uint64_t>((ra.rowoff + colc) * XB), xv[u]);
                ld_raw<RB * VEC, NT>(ra.rbase + static_cast<uint64_t>((ra.rowoff + colc) * RB), rv[u]);
            }
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            if (e0 + u < lds_chunks) {
                const uint32_t col = col0 + (CPT + e0 + u) * stride;
                float hx[VEC];
#pragma unroll
                for (int e = 0; e < VEC; ++e)
                    hx[e] = get_elem<XB, BF>(xv[u], e) + get_elem<RB, BF && RB == 2>(rv[u], e);
                if (ra.row_ok && col <= nlast) {
                    raw_t<RB * VEC> out;
                    pack_vec<RB, BF, VEC>(hx, out);
                    st_raw<RB * VEC, NT>(ra.rbase + static_cast<uint64_t>((ra.rowoff + col) * RB), out);
#pragma unroll
                    for (int e = 0; e < VEC; ++e) {
                        const double hd = static_cast<double>(hx[e]);
                        acc = __builtin_fma(hd, hd, acc);
                    }
                }
                float* slot = cache + static_cast<size_t>(e0 + u) * cache_step;
#pragma unroll
                for (int e = 0; e < VEC; ++e) slot[e] = hx[e];
            }
        }
    }
    // ---- streamed part, pass 1: sum only (default cache policy: pass 2 asks for the same lines again)
    for (uint32_t c0 = first_streamed; c0 < need; c0 += UNR) {
        raw_t<XB * VEC> xv[UNR];
        raw_t<RB * VEC> rv[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const uint32_t col = col0 + (c0 + u) * stride;
            if (c0 + u < need && col < n) {
                ld_raw<XB * VEC, false>(ra.xbase + static_cast<uint64_t>((ra.rowoff + col) * XB), xv[u]);
                ld_raw<RB * VEC, false>(ra.rbase + static_cast<uint64_t>((ra.rowoff + col) * RB), rv[u]);
            }
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const uint32_t col = col0 + (c0 + u) * stride;
            if (ra.row_ok && c0 + u < need && col < n) {
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const float hs = get_elem<XB, BF>(xv[u], e) + get_elem<RB, BF && RB == 2>(rv[u], e);
                    const double hd = static_cast<double>(hs);
                    acc = __builtin_fma(hd, hd, acc);
                }
            }
        }
    }

    const double ss = row_sum(acc, reduce, tpr, lane, ry, lds);
    const float rstd = rsqrt_to_f32(__builtin_fma(ss, inv_n, static_cast<double>(eps)));

    // ---- streamed part, pass 2, backwards
    for (uint32_t k = need; k > first_streamed;) {
        const uint32_t span_chunks = (k - first_streamed) < static_cast<uint32_t>(UNR) ? (k - first_streamed) : static_cast<uint32_t>(UNR);
        const uint32_t c0 = k - span_chunks;
        raw_t<XB * VEC> xv[UNR], wx[UNR];
        raw_t<RB * VEC> rv[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const uint32_t col = col0 + (c0 + u) * stride;
            if (static_cast<uint32_t>(u) < span_chunks && col < n) {
                ld_raw<XB * VEC, NT>(ra.xbase + static_cast<uint64_t>((ra.rowoff + col) * XB), xv[u]);
                ld_raw<RB * VEC, NT>(ra.rbase + static_cast<uint64_t>((ra.rowoff + col) * RB), rv[u]);
                ld_raw<XB * VEC>(wbase + static_cast<uint64_t>(col * XB), wx[u]);
            }
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const uint32_t col = col0 + (c0 + u) * stride;
            if (ra.row_ok && static_cast<uint32_t>(u) < span_chunks && col < n) {
                float hs[VEC], y[VEC];
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    hs[e] = get_elem<XB, BF>(xv[u], e) + get_elem<RB, BF && RB == 2>(rv[u], e);
                    const float t = hs[e] * rstd;
                    y[e] = t * get_elem<XB, BF>(wx[u], e);
                }
                raw_t<RB * VEC> rout;
                pack_vec<RB, BF, VEC>(hs, rout);
                st_raw<RB * VEC, NT>(ra.rbase + static_cast<uint64_t>((ra.rowoff + col) * RB), rout);
                raw_t<XB * VEC> yout;
                pack_vec<XB, BF, VEC>(y, yout);
                st_raw<XB * VEC, NT>(ra.xbase + static_cast<uint64_t>((ra.rowoff + col) * XB), yout);
            }
        }
        k = c0;
    }
    // ---- register part (weights fetched as they are needed: the registers are full of the row)
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
        const uint32_t col = col0 + static_cast<uint32_t>(c) * stride;
        raw_t<XB * VEC> wv;
        ld_raw<XB * VEC>(wbase + static_cast<uint64_t>((col < nlast ? col : nlast) * XB), wv);
        float y[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const float t = h[c][e] * rstd;
            y[e] = t * get_elem<XB, BF>(wv, e);
        }
        if (ra.row_ok && col <= nlast) {
            raw_t<XB * VEC> out;
            pack_vec<XB, BF, VEC>(y, out);
            st_raw<XB * VEC, NT>(ra.xbase + static_cast<uint64_t>((ra.rowoff + col) * XB), out);
        }
    }
    // ---- LDS part
    for (uint32_t e0 = 0; e0 < lds_chunks; e0 += UNR) {
        raw_t<XB * VEC> wx[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            if (e0 + u < lds_chunks) {
                const uint32_t col = col0 + (CPT + e0 + u) * stride;
                const uint32_t colc = col < nlast ? col : nlast;
                ld_raw<XB * VEC>(wbase + static_cast<uint64_t>(colc * XB), wx[u]);
            }
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            if (e0 + u < lds_chunks) {
                const uint32_t col = col0 + (CPT + e0 + u) * stride;
                const float* slot = cache + static_cast<size_t>(e0 + u) * cache_step;
                float y[VEC];
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const float t = slot[e] * rstd;
                    y[e] = t * get_elem<XB, BF>(wx[u], e);
                }
                if (ra.row_ok && col <= nlast) {
                    raw_t<XB * VEC> out;
                    pack_vec<XB, BF, VEC>(y, out);
                    st_raw<XB * VEC, NT>(ra.xbase + static_cast<uint64_t>((ra.rowoff + col) * XB), out);
                }
            }
        }
    }
}

// Aligned-span form, for rows whose byte length is not a whole number of cache lines (N = 1000:
// 2000 and 4000 bytes).  In the forms above a wave's access starts wherever its row starts, so
// every access straddles lines that a neighbouring wave - often of another workgroup - also
// touches, and partly written lines have to be merged on the way to memory.  Here a workgroup
// owns blockDim.y consecutive rows whose combined length IS a whole number of lines (the host
// checks that), treats them as one flat span of 16-byte pieces (VEC elements; a piece never
// straddles two rows because VEC divides N) and maps piece p = c * T + t to thread t: every
// wave-wide access is one aligned, contiguous kilobyte (half of that for the 16-bit stream of
// the mixed format) and every line is written whole by one instruction.  The price is a
// segmented reduction, since row boundaries fall inside waves: each piece's sum of squares
// goes to LDS, one wave per row adds that row's pieces (strided, then the cross-lane
// sum), and the row's rstd is left in LDS for every piece of the row.
// LDS: T * CPT doubles (piece sums), then blockDim.y floats (rstd per row).
template <int DT, int VEC, int CPT, int UNR, bool NT, bool DEFER>
__device__ __forceinline__ void addrms_span_body(void* __restrict__ xp, void* __restrict__ rp,
                                                 const void* __restrict__ wp, float eps, double inv_n,
                                                 int64_t M, int32_t N, uint32_t flags, int32_t reduce,
                                                 uint32_t nblocks)
{
    using T_ = dt_traits<DT>;
    constexpr int XB = T_::XB, RB = T_::RB;
    constexpr bool BF = T_::BF;
    static_assert(VEC * XB <= 16 && VEC * RB <= 16, "one access per stream and piece");
    extern __shared__ double lds[];
    (void)reduce; (void)nblocks;

    const uint32_t T = blockDim.x * blockDim.y, R = blockDim.y;
    const uint32_t t = threadIdx.y * blockDim.x + threadIdx.x;
    uint32_t blk = blockIdx.x;
    if (flags & FLAG_XCD_CONTIG) blk = xcd_contiguous(blk, gridDim.x);
    const int64_t row0 = static_cast<int64_t>(blk) * R;
    const int64_t left = M - row0;
    const uint32_t rows_here = left < static_cast<int64_t>(R) ? static_cast<uint32_t>(left) : R;
    const uint32_t P = static_cast<uint32_t>(N) / VEC;            // pieces per row
    const uint32_t S = rows_here * P;                             // pieces of this span
    char* xspan = static_cast<char*>(xp) + row0 * N * XB;
    char* rspan = static_cast<char*>(rp) + row0 * N * RB;
    const char* wbase = static_cast<const char*>(wp);
    double* part = lds;
    float* rstd_s = reinterpret_cast<float*>(lds + static_cast<size_t>(T) * CPT);

    float h[CPT][VEC];
#pragma unroll
    for (int g = 0; g < CPT; g += UNR) {
        raw_t<XB * VEC> xv[UNR];
        raw_t<RB * VEC> rv[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            if (g + u < CPT) {
                const uint32_t p = static_cast<uint32_t>(g + u) * T + t;
                const uint32_t pc = p < S ? p : S - 1u;           // idle threads re-read the last piece
                ld_raw<XB * VEC, NT>(xspan + static_cast<uint64_t>(pc * (VEC * XB)), xv[u]);
                ld_raw<RB * VEC, NT>(rspan + static_cast<uint64_t>(pc * (VEC * RB)), rv[u]);
            }
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            if (g + u < CPT) {
                const int c = g + u;
                const uint32_t p = static_cast<uint32_t>(c) * T + t;
#pragma unroll
                for (int e = 0; e < VEC; ++e)
                    h[c][e] = get_elem<XB, BF>(xv[u], e) + get_elem<RB, BF && RB == 2>(rv[u], e);
                if (p < S) {
                    if constexpr (!DEFER) {
                        raw_t<RB * VEC> out;
                        pack_vec<RB, BF, VEC>(h[c], out);
                        st_raw<RB * VEC, NT>(rspan + static_cast<uint64_t>(p * (VEC * RB)), out);
                    }
                    double acc = 0.0;
#pragma unroll
                    for (int e = 0; e < VEC; ++e) {
                        const double hd = static_cast<double>(h[c][e]);
                        acc = __builtin_fma(hd, hd, acc);
                    }
                    part[p] = acc;
                }
            }
        }
        if (g + UNR < CPT) __builtin_amdgcn_sched_barrier(0);
    }
    wg_sync_lds();
    {
        const uint32_t wv = t >> 6, l = t & 63u, nw = T >> 6;
        for (uint32_t k = wv; k < rows_here; k += nw) {           // uniform over the wave
            double s = 0.0;
            for (uint32_t j = l; j < P; j += 64u) s += part[k * P + j];
            s = wave_total(s);
            if (l == 0u) rstd_s[k] = rsqrt_to_f32(__builtin_fma(s, inv_n, static_cast<double>(eps)));
        }
    }
    wg_sync_lds();

    uint32_t prow[CPT];
    raw_t<XB * VEC> wv_[CPT];
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
        const uint32_t p = static_cast<uint32_t>(c) * T + t;
        const uint32_t pc = p < S ? p : S - 1u;
        prow[c] = pc / P;
        ld_raw<XB * VEC>(wbase + static_cast<uint64_t>((pc - prow[c] * P) * (VEC * XB)), wv_[c]);
    }
    if constexpr (DEFER) {
#pragma unroll
        for (int c = 0; c < CPT; ++c) {
            const uint32_t p = static_cast<uint32_t>(c) * T + t;
            if (p < S) {
                raw_t<RB * VEC> out;
                pack_vec<RB, BF, VEC>(h[c], out);
                st_raw<RB * VEC, NT>(rspan + static_cast<uint64_t>(p * (VEC * RB)), out);
            }
        }
    }
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
        const uint32_t p = static_cast<uint32_t>(c) * T + t;
        const float rstd = rstd_s[prow[c]];
        float y[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const float tt = h[c][e] * rstd;
            y[e] = tt * get_elem<XB, BF>(wv_[c], e);
        }
        if (p < S) {
            raw_t<XB * VEC> out;
            pack_vec<XB, BF, VEC>(y, out);
            st_raw<XB * VEC, NT>(xspan + static_cast<uint64_t>(p * (VEC * XB)), out);
        }
    }
}

}  // namespace addrms
