// Device-side template of merge_attn_states for gfx950, the third kernel put through the
// tuner (Section 4, "Kernels"; its shapes are (n, h, d) = tokens x heads x head size).
//
// Per row (one token and head) with partial outputs v_a, v_b of d lanes and their
// log-sum-exp scores s_a, s_b:
//     m = max(s_a, s_b);  e_a = exp(s_a - m);  e_b = exp(s_b - m)
//     v_out = (e_a v_a + e_b v_b) / (e_a + e_b);   s_out = m + log(e_a + e_b)
//
// Same knob set as silu_and_mul (no reduction: every lane of a row reads the two
// scores itself; the loads hit one address per row).  Rows are short (d = 128 or
// 256), so a row is 8 to 32 lanes and a wave carries several rows.  Arithmetic: fp32
// with the hardware base-2 exponential, logarithm and reciprocal; v_out is rounded
// once, to nearest even, into the storage format.
#pragma once
#include "addrms_kernel.h"

namespace addrms {

template <int DT, int VEC, int CPT, int UNR, bool NT>
__device__ __forceinline__ void mergestates_body(const void* __restrict__ vap, const float* __restrict__ sap,
                                                 const void* __restrict__ vbp, const float* __restrict__ sbp,
                                                 void* __restrict__ vop, float* __restrict__ sop, int64_t rows,
                                                 int32_t d, uint32_t flags, uint32_t nblocks)
{
    using T = dt_traits<DT>;
    constexpr int ES = T::XB;
    constexpr bool BF = T::BF;
    constexpr float kLog2e = 1.44269504088896340736f, kLn2 = 0.69314718055994530942f;
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
        asm volatile("" : "+v"(col0));
        const int64_t row0 = static_cast<int64_t>(blk) * rpw;
        const int64_t left = rows - row0;                       // >= 1
        const bool row_ok = static_cast<int64_t>(ry) < left;
        const uint32_t ryc = row_ok ? ry : static_cast<uint32_t>(left - 1);
        const char* a_base = static_cast<const char*>(vap) + row0 * d * ES;     // wave-uniform bases
        const char* b_base = static_cast<const char*>(vbp) + row0 * d * ES;
        char* o_base = static_cast<char*>(vop) + row0 * d * ES;
        const uint32_t off = ryc * ud;                                           // elements, fits 32 bits
        const float sa = sap[row0 + ryc], sb = sbp[row0 + ryc];

        raw_t<ES * VEC> av[UNR], bv[UNR];
        float wa = 0.0f, wb = 0.0f;
#pragma unroll
        for (int g0 = 0; g0 < CPT; g0 += UNR) {
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                if (g0 + u < CPT) {
                    const uint32_t col = col0 + static_cast<uint32_t>(g0 + u) * stride;
                    const uint32_t colc = col < nlast ? col : nlast;
                    ld_raw<ES * VEC, NT>(a_base + static_cast<uint64_t>((off + colc) * ES), av[u]);
                    ld_raw<ES * VEC, NT>(b_base + static_cast<uint64_t>((off + colc) * ES), bv[u]);
                }
            }
            if (g0 == 0) {
                // the row's two weights, while the first loads are in flight
                const float m = sa > sb ? sa : sb;
                const float ea = __builtin_amdgcn_exp2f((sa - m) * kLog2e);
                const float eb = __builtin_amdgcn_exp2f((sb - m) * kLog2e);
                const float denom = ea + eb;
                const float inv = __builtin_amdgcn_rcpf(denom);
                wa = ea * inv;
                wb = eb * inv;
                if (row_ok && lane == 0) sop[row0 + ryc] = m + __builtin_amdgcn_logf(denom) * kLn2;
            }
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                if (g0 + u < CPT) {
                    const uint32_t col = col0 + static_cast<uint32_t>(g0 + u) * stride;
                    float y[VEC];
#pragma unroll
                    for (int e = 0; e < VEC; ++e) {
                        const float tb = wb * get_elem<ES, BF>(bv[u], e);
                        y[e] = __builtin_fmaf(wa, get_elem<ES, BF>(av[u], e), tb);
                    }
                    if (row_ok && col <= nlast) {
                        raw_t<ES * VEC> out;
                        pack_vec<ES, BF, VEC>(y, out);
                        st_raw<ES * VEC, NT>(o_base + static_cast<uint64_t>((off + col) * ES), out);
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
