// Parameter-space merge and its two adjoints as small-K MFMA contractions
// (gfx950, bf16 operands, fp32 accumulation).
//
// Paper Eq. 2: theta_bar(s) = sum_e w[s,e] * theta_e for every segment s; by
// the chain rule dtheta_e = sum_s w[s,e] * dtheta_bar(s) and
// dw[s,e] = <theta_e, dtheta_bar(s)>.  For a rectangle of an expert matrix
// (rows r0..r0+nr, columns c0..c0+nc) these are three thin GEMMs:
//   merge:   slab[S, n]  = w[S, E]     * stack[E, n]        (K = E)
//   scatter: dW[E, n]    = w^T[E, S]   * gslab[S, n]        (K = S)
//   dots:    dw[S, E]   += gslab[S, n] * stack[E, n]^T      (K = n)
// The passes are HBM-bound; the vector ALUs could not keep up with the E (or
// S) multiply-adds per element, so all three run on the matrix cores.
//
// Work unit of a wavefront: 32 consecutive 16-byte chunks (256 elements) of the
// rectangle.  A lane loads one chunk per expert (or segment) row, i.e. eight
// consecutive elements of ONE row, while the MFMA wants eight consecutive K
// (rows) of ONE element; the 8x8 transposition is done in registers with byte
// permutes.  Routing weights enter as bf16 hi + lo pairs (two MFMAs), which
// keeps their relative error near 2^-17 instead of 2^-9.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_bf16.h"

namespace lory {
namespace ms {

using gemm::bf16x8;
using gemm::f32x16;

// A rectangle of one expert matrix inside the [E, rows, pitch] stack.
struct Rect {
    long expert_stride;  // elements between experts
    int pitch;           // elements between rows of the matrix
    int r0, c0, nr, nc;  // rectangle; nc % 8 == 0
};

__device__ __forceinline__ long rect_offset(const Rect &rc, int q)
{
    const int cpr = rc.nc >> 3;
    const int r = q / cpr, c = (q - r * cpr) << 3;
    return (long)(rc.r0 + r) * rc.pitch + rc.c0 + c;
}

union Frag {
    uint4 u;
    uint32_t w[4];
    bf16x8 v;
};

// out[j] holds, for element j of the chunk, rows 0..7 packed as 8 bf16.
__device__ __forceinline__ void transpose8x8(const Frag (&in)[8], Frag (&out)[8])
{
#pragma unroll
    for (int j = 0; j < 8; ++j) {
#pragma unroll
        for (int ip = 0; ip < 4; ++ip) {
            const uint32_t a = in[2 * ip].w[j >> 1];
            const uint32_t b = in[2 * ip + 1].w[j >> 1];
            // v_perm_b32: result bytes picked from {b (bytes 4..7), a (bytes 0..3)}
            out[j].w[ip] = (j & 1) ? __builtin_amdgcn_perm(b, a, 0x07060302u)
                                   : __builtin_amdgcn_perm(b, a, 0x05040100u);
        }
    }
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    return (uint32_t)gemm::float_to_bf16_bits(lo) | ((uint32_t)gemm::float_to_bf16_bits(hi) << 16);
}

// Eight fp32 routing weights -> bf16 hi and lo operand fragments.
__device__ __forceinline__ void split_hi_lo(const float (&v)[8], Frag &hi, Frag &lo)
{
    float h[8], l[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const uint16_t hb = gemm::float_to_bf16_bits(v[i]);
        h[i] = gemm::bf16_bits_to_float(hb);
        l[i] = v[i] - h[i];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        hi.w[i] = pack_bf16(h[2 * i], h[2 * i + 1]);
        lo.w[i] = pack_bf16(l[2 * i], l[2 * i + 1]);
    }
}

// ------------------------------------------------------------------ merge

struct MergeParams {
    const float *w;         // [S, E]
    int S, E;
    const uint16_t *stack;  // expert stack base of this matrix
    Rect rc;
    uint16_t *slab;         // [S][nr*nc]
    long seg_stride;
};

// KS = ceil(E / 16).  grid.x workgroups of 256 threads stride over the units.
// Dynamic LDS: ceil(S/32) * KS * 2 * 64 * 16 bytes (routing-weight operands).
template <int KS>
__global__ __launch_bounds__(256) void merge_kernel(const MergeParams p)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    uint4 *wtab = reinterpret_cast<uint4 *>(smem);  // [mb][ks][hi/lo][lane]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ln = lane & 31, h = lane >> 5;
    const int MB = (p.S + 31) >> 5;

    for (int idx = tid; idx < MB * KS * 64; idx += 256) {
        const int l = idx & 63, ks = (idx >> 6) % KS, mb = (idx >> 6) / KS;
        const int seg = mb * 32 + (l & 31);
        float v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int e = 16 * ks + 8 * (l >> 5) + i;
            v[i] = (seg < p.S && e < p.E) ? p.w[(size_t)seg * p.E + e] : 0.f;
        }
        Frag hi, lo;
        split_hi_lo(v, hi, lo);
        wtab[((mb * KS + ks) * 2 + 0) * 64 + l] = hi.u;
        wtab[((mb * KS + ks) * 2 + 1) * 64 + l] = lo.u;
    }
    __syncthreads();

    const int Q = (p.rc.nr * p.rc.nc) >> 3;
    const int units = (Q + 31) >> 5;
    const int stride = gridDim.x * 4;

    Frag R[KS][8];
    auto load_unit = [&](int unit) {
        const int q = unit * 32 + ln;
        const bool ok = q < Q;
        const long off = ok ? rect_offset(p.rc, q) : 0;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int e = 16 * ks + 8 * h + i;
                if (ok && e < p.E)
                    R[ks][i].u = *reinterpret_cast<const uint4 *>(p.stack + (size_t)e * p.rc.expert_stride + off);
                else
                    R[ks][i].u = make_uint4(0, 0, 0, 0);
            }
    };

    int unit = blockIdx.x * 4 + wave;
    if (unit < units) load_unit(unit);
    for (; unit < units; unit += stride) {
        Frag P[KS][8];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) transpose8x8(R[ks], P[ks]);
        if (unit + stride < units) load_unit(unit + stride);  // prefetch behind the MFMAs

        const int q = unit * 32 + ln;
        for (int mb = 0; mb < MB; ++mb) {
            f32x16 acc[8];
#pragma unroll
            for (int j = 0; j < 8; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                Frag whi, wlo;
                whi.u = wtab[((mb * KS + ks) * 2 + 0) * 64 + lane];
                wlo.u = wtab[((mb * KS + ks) * 2 + 1) * 64 + lane];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(whi.v, P[ks][j].v, acc[j], 0, 0, 0);
                    acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wlo.v, P[ks][j].v, acc[j], 0, 0, 0);
                }
            }
            if (q < Q) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int seg = mb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                    if (seg < p.S) {
                        uint4 o;
                        o.x = pack_bf16(acc[0][r], acc[1][r]);
                        o.y = pack_bf16(acc[2][r], acc[3][r]);
                        o.z = pack_bf16(acc[4][r], acc[5][r]);
                        o.w = pack_bf16(acc[6][r], acc[7][r]);
                        *reinterpret_cast<uint4 *>(p.slab + (size_t)seg * p.seg_stride + (size_t)q * 8) = o;
                    }
                }
            }
        }
    }
}

// ------------------------------------------------------ scatter + dots

struct ScatterParams {
    const float *w;          // [S, E]
    int S, E;
    const uint16_t *gslab;   // per-segment weight gradients [S][nr*nc] (bf16)
    long seg_stride;
    const uint16_t *stack;   // expert stack base of this matrix (for the inner products)
    void *dW;                // gradient stack base of this matrix, addressed like `stack`
    Rect rc;
    int grad_f32;            // dW is fp32 (else bf16)
    int accumulate;          // add to dW instead of overwriting it
    float *partials;         // [gridDim.x * 4][SB*32][EB*32] per-wave router-weight partial sums
    int partials_add;        // add to the existing partials instead of overwriting them
};

// NACC = SBn * EBS 32x32 router-weight accumulator blocks, SBn >= ceil(S/32),
// EBS >= ceil(E/32).  grid.x workgroups of 256 threads stride over the units.
// Dynamic LDS: ceil(E/32) * ceil(S/16) * 2 * 64 * 16 bytes (transposed
// routing-weight operands).
template <int NACC, int EBS>
__global__ __launch_bounds__(256) void scatter_kernel(const ScatterParams p)
{
    constexpr int SBn = NACC / EBS;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    uint4 *wtab = reinterpret_cast<uint4 *>(smem);  // [eb][kb][hi/lo][lane]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ln = lane & 31, h = lane >> 5;
    const int EB = (p.E + 31) >> 5, KB = (p.S + 15) >> 4;

    for (int idx = tid; idx < EB * KB * 64; idx += 256) {
        const int l = idx & 63, kb = (idx >> 6) % KB, eb = (idx >> 6) / KB;
        const int e = eb * 32 + (l & 31);
        float v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int seg = 16 * kb + 8 * (l >> 5) + i;
            v[i] = (seg < p.S && e < p.E) ? p.w[(size_t)seg * p.E + e] : 0.f;
        }
        Frag hi, lo;
        split_hi_lo(v, hi, lo);
        wtab[((eb * KB + kb) * 2 + 0) * 64 + l] = hi.u;
        wtab[((eb * KB + kb) * 2 + 1) * 64 + l] = lo.u;
    }
    __syncthreads();

    const int Q = (p.rc.nr * p.rc.nc) >> 3;
    const int units = (Q + 31) >> 5;
    const int stride = gridDim.x * 4;

    f32x16 dots[NACC];
#pragma unroll
    for (int a = 0; a < NACC; ++a)
#pragma unroll
        for (int r = 0; r < 16; ++r) dots[a][r] = 0.f;

    for (int unit = blockIdx.x * 4 + wave; unit < units; unit += stride) {
        const int q = unit * 32 + ln;
        const bool ok = q < Q;

        // ---- dW[e] = sum_s w[s,e] * gslab[s]   (K = segments, 16 per step)
        f32x16 acc[EBS][8];
#pragma unroll
        for (int eb = 0; eb < EBS; ++eb)
#pragma unroll
            for (int j = 0; j < 8; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[eb][j][r] = 0.f;
        for (int kb = 0; kb < KB; ++kb) {
            Frag Rg[8], P[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int seg = 16 * kb + 8 * h + i;
                if (ok && seg < p.S)
                    Rg[i].u = *reinterpret_cast<const uint4 *>(p.gslab + (size_t)seg * p.seg_stride + (size_t)q * 8);
                else
                    Rg[i].u = make_uint4(0, 0, 0, 0);
            }
            transpose8x8(Rg, P);
#pragma unroll
            for (int eb = 0; eb < EBS; ++eb) {
                if (eb < EB) {
                    Frag whi, wlo;
                    whi.u = wtab[((eb * KB + kb) * 2 + 0) * 64 + lane];
                    wlo.u = wtab[((eb * KB + kb) * 2 + 1) * 64 + lane];
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        acc[eb][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(whi.v, P[j].v, acc[eb][j], 0, 0, 0);
                        acc[eb][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wlo.v, P[j].v, acc[eb][j], 0, 0, 0);
                    }
                }
            }
        }
        if (ok) {
            const long off = rect_offset(p.rc, q);
#pragma unroll
            for (int eb = 0; eb < EBS; ++eb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int e = eb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                    if (e >= p.E) continue;
                    float v[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) v[j] = acc[eb][j][r];
                    if (p.grad_f32) {
                        float4 *dst = reinterpret_cast<float4 *>(reinterpret_cast<float *>(p.dW) +
                                                                 (size_t)e * p.rc.expert_stride + off);
                        float4 o0 = make_float4(v[0], v[1], v[2], v[3]);
                        float4 o1 = make_float4(v[4], v[5], v[6], v[7]);
                        if (p.accumulate) {
                            const float4 c0 = dst[0], c1 = dst[1];
                            o0.x += c0.x; o0.y += c0.y; o0.z += c0.z; o0.w += c0.w;
                            o1.x += c1.x; o1.y += c1.y; o1.z += c1.z; o1.w += c1.w;
                        }
                        dst[0] = o0;
                        dst[1] = o1;
                    } else {
                        uint4 *dst = reinterpret_cast<uint4 *>(reinterpret_cast<uint16_t *>(p.dW) +
                                                               (size_t)e * p.rc.expert_stride + off);
                        if (p.accumulate) {
                            const uint4 c = *dst;
                            const uint32_t cw[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                v[2 * i] += __uint_as_float(cw[i] << 16);
                                v[2 * i + 1] += __uint_as_float(cw[i] & 0xffff0000u);
                            }
                        }
                        uint4 o;
                        o.x = pack_bf16(v[0], v[1]);
                        o.y = pack_bf16(v[2], v[3]);
                        o.z = pack_bf16(v[4], v[5]);
                        o.w = pack_bf16(v[6], v[7]);
                        *dst = o;
                    }
                }
        }

        // ---- dw[s,e] += <stack[e], gslab[s]> over this unit  (K = elements, 16 per step)
        const int q0 = unit * 32;
#pragma unroll 4
        for (int ks = 0; ks < 16; ++ks) {
            const int qq = q0 + 2 * ks + h;
            const bool okq = qq < Q;
            const long off2 = okq ? rect_offset(p.rc, qq) : 0;
            Frag bfr[EBS];
#pragma unroll
            for (int eb = 0; eb < EBS; ++eb) {
                const int e = eb * 32 + ln;
                if (okq && e < p.E)
                    bfr[eb].u = *reinterpret_cast<const uint4 *>(p.stack + (size_t)e * p.rc.expert_stride + off2);
                else
                    bfr[eb].u = make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int sb = 0; sb < SBn; ++sb) {
                const int seg = sb * 32 + ln;
                Frag af;
                if (okq && seg < p.S)
                    af.u = *reinterpret_cast<const uint4 *>(p.gslab + (size_t)seg * p.seg_stride + (size_t)qq * 8);
                else
                    af.u = make_uint4(0, 0, 0, 0);
#pragma unroll
                for (int eb = 0; eb < EBS; ++eb)
                    dots[sb * EBS + eb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af.v, bfr[eb].v,
                                                                                dots[sb * EBS + eb], 0, 0, 0);
            }
        }
    }

    // per-wave partial sums; a later kernel adds them up in slot order
    const size_t slot = (size_t)blockIdx.x * 4 + wave;
    float *part = p.partials + slot * (SBn * 32) * (EBS * 32);
#pragma unroll
    for (int a = 0; a < NACC; ++a)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int seg = (a / EBS) * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
            const int e = (a % EBS) * 32 + ln;
            float *dst = part + (size_t)seg * (EBS * 32) + e;
            *dst = p.partials_add ? (*dst + dots[a][r]) : dots[a][r];
        }
}

}  // namespace ms
}  // namespace lory
