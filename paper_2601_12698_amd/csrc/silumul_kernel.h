// Device-side template of silu_and_mul for gfx950, the second kernel put through
// the same tuner (the paper evaluates three serving kernels, Section 4, "Kernels").
//
//   out[i, j] = silu(x[i, j]) * x[i, d + j],   silu(g) = g / (1 + exp(-g)),   j < d
//
// Same knob set as the add+RMSNorm template minus the reduction: VEC, CPT (chunks
// per thread along a row of d outputs), UNR (chunks whose loads are in flight),
// NT (non-temporal policy) are compile-time; threads_per_row, rows_per_wg, the
// XCD-contiguous mapping, the occupancy cap and the persistent grid are launch-time.
//
// Arithmetic: fp32; exp through the hardware base-2 exponential, the quotient
// through the hardware reciprocal (a few fp32 ulps in all); one rounding to
// nearest-even into the storage format.  HBM-bound: 6 bytes per output for
// 16-bit storage against roughly 15 lane-cycles of arithmetic.
#pragma once
#include "addrms_kernel.h"

namespace addrms {

__device__ __forceinline__ float silu_times(float g, float u)
{
    const float e = __builtin_amdgcn_exp2f(g * -1.44269504088896340736f);   // exp(-g)
    const float s = g * __builtin_amdgcn_rcpf(1.0f + e);
    return s * u;
}

template <int DT, int VEC, int CPT, int UNR, bool NT>
__device__ __forceinline__ void silumul_body(const void* __restrict__ xp, void* __restrict__ op, int64_t M,
                                             int32_t d, uint32_t flags, uint32_t nblocks)
{
    using T = dt_traits<DT>;
    constexpr int ES = T::XB;
    constexpr bool BF = T::BF;
    const uint32_t tpr = blockDim.x, rpw = blockDim.y;
    const uint32_t lane = threadIdx.x, ry = threadIdx.y;
    uint32_t blk = blockIdx.x;
    if (flags & FLAG_XCD_CONTIG) blk = xcd_contiguous(blk, gridDim.x);
    const uint32_t col_first = lane * VEC;
    const uint32_t stride = tpr * VEC;
    const uint32_t nlast = static_cast<uint32_t>(d) - VEC;
    const uint32_t ud = static_cast<uint32_t>(d);

    for (;;) {
        uint32_t col0 = col_first;
        asm volatile("" : "+v"(col0));          // keep per-chunk offsets out of the loop-carried registers
        const int64_t row0 = static_cast<int64_t>(blk) * rpw;
        const int64_t left = M - row0;                          // >= 1
        const bool row_ok = static_cast<int64_t>(ry) < left;
        const uint32_t ryc = row_ok ? ry : static_cast<uint32_t>(left - 1);
        const char* in_base = static_cast<const char*>(xp) + row0 * 2 * d * ES;   // wave-uniform
        char* out_base = static_cast<char*>(op) + row0 * d * ES;
        const uint32_t in_off = ryc * 2u * ud, out_off = ryc * ud;              // elements, fit 32 bits

#pragma unroll
        for (int g0 = 0; g0 < CPT; g0 += UNR) {
            raw_t<ES * VEC> gv[UNR], uv[UNR];
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                if (g0 + u < CPT) {
                    const uint32_t col = col0 + static_cast<uint32_t>(g0 + u) * stride;
                    const uint32_t colc = col < nlast ? col : nlast;          // tail lanes re-read valid data
                    ld_raw<ES * VEC, NT>(in_base + static_cast<uint64_t>((in_off + colc) * ES), gv[u]);
                    ld_raw<ES * VEC, NT>(in_base + static_cast<uint64_t>((in_off + ud + colc) * ES), uv[u]);
                }
            }
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                if (g0 + u < CPT) {
                    const uint32_t col = col0 + static_cast<uint32_t>(g0 + u) * stride;
                    float y[VEC];
#pragma unroll
                    for (int e = 0; e < VEC; ++e)
                        y[e] = silu_times(get_elem<ES, BF>(gv[u], e), get_elem<ES, BF>(uv[u], e));
                    if (row_ok && col <= nlast) {
                        raw_t<ES * VEC> out;
                        pack_vec<ES, BF, VEC>(y, out);
                        st_raw<ES * VEC, NT>(out_base + static_cast<uint64_t>((out_off + col) * ES), out);
                    }
                }
            }
            if (g0 + UNR < CPT) __builtin_amdgcn_sched_barrier(0);
        }
        const uint32_t next = blk + gridDim.x;      // a persistent grid walks several row blocks
        if (next >= nblocks) break;
        blk = next;
    }
}

}  // namespace addrms
