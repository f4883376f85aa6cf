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
    return gemm::cvt_pk_bf16(lo, hi);
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

    // Up to 32 experts the next unit is fetched behind the MFMAs of the current one; with more, the
    // registers of a second set of chunks do not exist (the kernel would spill), so a unit is
    // fetched when its turn comes.
    constexpr bool kPrefetch = KS <= 2;
    int unit = blockIdx.x * 4 + wave;
    if (kPrefetch && unit < units) load_unit(unit);
    for (; unit < units; unit += stride) {
        if constexpr (!kPrefetch) load_unit(unit);
        Frag P[KS][8];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) transpose8x8(R[ks], P[ks]);
        if constexpr (kPrefetch) {
            if (unit + stride < units) load_unit(unit + stride);
        }

        const int q = unit * 32 + ln;
        // JH column elements of a chunk at a time: all 8 (16-byte stores), or 4 (8-byte stores) when the
        // chunks of more than 32 experts leave too few registers for 8 accumulator blocks
        constexpr int JH = kPrefetch ? 8 : 4;
        for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
            for (int j0 = 0; j0 < 8; j0 += JH) {
                f32x16 acc[JH];
#pragma unroll
                for (int j = 0; j < JH; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    Frag whi, wlo;
                    whi.u = wtab[((mb * KS + ks) * 2 + 0) * 64 + lane];
                    wlo.u = wtab[((mb * KS + ks) * 2 + 1) * 64 + lane];
#pragma unroll
                    for (int j = 0; j < JH; ++j) {
                        acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(whi.v, P[ks][j0 + j].v, acc[j], 0, 0, 0);
                        acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wlo.v, P[ks][j0 + j].v, acc[j], 0, 0, 0);
                    }
                }
                if (q < Q) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int seg = mb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                        if (seg < p.S) {
                            uint16_t *dst = p.slab + (size_t)seg * p.seg_stride + (size_t)q * 8 + j0;
                            if constexpr (JH == 8) {
                                uint4 o;
                                o.x = pack_bf16(acc[0][r], acc[1][r]);
                                o.y = pack_bf16(acc[2][r], acc[3][r]);
                                o.z = pack_bf16(acc[4][r], acc[5][r]);
                                o.w = pack_bf16(acc[6][r], acc[7][r]);
                                *reinterpret_cast<uint4 *>(dst) = o;
                            } else {
                                uint2 o;
                                o.x = pack_bf16(acc[0][r], acc[1][r]);
                                o.y = pack_bf16(acc[2][r], acc[3][r]);
                                *reinterpret_cast<uint2 *>(dst) = o;
                            }
                        }
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
    int e0;                  // first expert of the window of up to 32 experts this launch handles
    const uint16_t *gslab;   // per-segment weight gradients [S][nr*nc] (bf16)
    long seg_stride;
    const uint16_t *stack;   // expert stack base of this matrix (for the inner products)
    void *dW;                // gradient stack base of this matrix, addressed like `stack`
    Rect rc;
    int grad_f32;            // dW is fp32 (else bf16)
    int accumulate;          // add to dW instead of overwriting it
    float *partials;         // [gridDim.x][KBM*16][pcols] per-workgroup router-weight partial sums
    int pcols;               // columns of a partials row (>= E)
    int partials_add;        // add to the existing partials instead of overwriting them
};

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kDotPitch = 272;  // bytes per segment row of a wave's LDS staging area (256 + 16)

// One launch handles the experts e0 .. e0+31 (clipped to E).
//   KBM  >= ceil(S / 16): static bound on the 16-segment K blocks
//   EB16 =  ceil(window / 16): 16-expert blocks of the router-weight accumulators (1 or 2)
// Work unit of a wavefront here: 16 consecutive 16-byte chunks (128 elements).  Lane
// (chunk c = lane & 15, element half hh = (lane >> 4) & 1, segment half sh = lane >> 5) handles
// elements 4hh..4hh+3 of chunk c: it loads them (8 bytes) from 8 segments per block of 16
// segments, transposes them in registers into "8 segments of one element" (the B operand of
// the scatter MFMA, K = segments, column = (c, hh)), and parks them in the wave's LDS area, from
// where the inner-product MFMAs (16x16x32, K = elements) read them row-per-lane; every gradient
// byte is fetched from memory once.  The small unit keeps a wave under 256 registers, so two
// workgroups share a CU and hide each other's memory latency.
// Per unit a wave
//   (1) loads the window's expert chunks once (B operand of the inner products),
//   (2) walks the segments 16 at a time (next block's loads in flight behind the MFMAs),
//   (3) writes 32 experts x 128 elements of expert gradients.
// Dynamic LDS: the larger of KB * 2 * 64 * 16 bytes of routing-weight operands + 4 * 16 * kDotPitch
// (+ 4 * EB16 * 4096 when the expert chunks are parked, below) and 4 * KBM * EB16 * 1024 bytes for the
// final reduction of the router-weight accumulators.
// Two workgroups per CU wherever a wave stays under 256 registers: up to 8 blocks of router-weight
// accumulators, and 16 blocks (129-256 segments with at most 16 experts: the short-segment shapes,
// 3.7 -> 4.9 TB/s; 65-128 segments with 17-32 experts) with the unit's expert chunks parked in LDS
// instead of 16 or 32 registers.
template <int KBM, int EB16>
constexpr bool scatter_parks_experts() { return KBM * EB16 == 16; }

template <int KBM, int EB16>
__global__ __launch_bounds__(256, (KBM * EB16 <= 8 || scatter_parks_experts<KBM, EB16>()) ? 2 : 1) void scatter_kernel(const ScatterParams p)
{
    constexpr bool kParkB = scatter_parks_experts<KBM, EB16>();
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, hh = (lane >> 4) & 1, sh = lane >> 5;
    const int KB = (p.S + 15) >> 4;
    uint4 *wtab = reinterpret_cast<uint4 *>(smem);  // [kb][hi/lo][lane]
    char *park = smem + (size_t)KB * 2 * 64 * 16 + wave * (16 * kDotPitch);
    char *parkB = smem + (size_t)KB * 2 * 64 * 16 + 4 * (16 * kDotPitch) + wave * (EB16 * 4096);   // kParkB only
    const int Ewin = (p.E - p.e0 < 32) ? (p.E - p.e0) : 32;

    for (int idx = tid; idx < KB * 64; idx += 256) {
        const int l = idx & 63, kb = idx >> 6;
        const int e = l & 31;
        float v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int seg = 16 * kb + 8 * (l >> 5) + i;
            v[i] = (seg < p.S && e < Ewin) ? p.w[(size_t)seg * p.E + p.e0 + e] : 0.f;
        }
        Frag hi, lo;
        split_hi_lo(v, hi, lo);
        wtab[(kb * 2 + 0) * 64 + l] = hi.u;
        wtab[(kb * 2 + 1) * 64 + l] = lo.u;
    }
    __syncthreads();

    const int Q = (p.rc.nr * p.rc.nc) >> 3;
    const int units = (Q + 15) >> 4;
    const int stride = gridDim.x * 4;
    const uint16_t *stack = p.stack + (size_t)p.e0 * p.rc.expert_stride;

    f32x4 dots[KBM][EB16];
#pragma unroll
    for (int a = 0; a < KBM; ++a)
#pragma unroll
        for (int b = 0; b < EB16; ++b)
#pragma unroll
            for (int r = 0; r < 4; ++r) dots[a][b][r] = 0.f;

    for (int unit = blockIdx.x * 4 + wave; unit < units; unit += stride) {
        const int q = unit * 16 + c;
        const bool ok = q < Q;

        // expert chunks of the window: lane (n = lane & 15, chunk 4*kq + (lane >> 4))
        Frag Bst[EB16][4];
#pragma unroll
        for (int kq = 0; kq < 4; ++kq) {
            const int qq = unit * 16 + 4 * kq + (lane >> 4);
            const bool okq = qq < Q;
            const long off2 = okq ? rect_offset(p.rc, qq) : 0;
#pragma unroll
            for (int b = 0; b < EB16; ++b) {
                const int e = b * 16 + (lane & 15);
                if (okq && e < Ewin)
                    Bst[b][kq].u = *reinterpret_cast<const uint4 *>(stack + (size_t)e * p.rc.expert_stride + off2);
                else
                    Bst[b][kq].u = make_uint4(0, 0, 0, 0);
            }
        }
        if constexpr (kParkB) {
            // (the previous unit's reads of this area have returned: LDS operations of a wave stay in order)
#pragma unroll
            for (int b = 0; b < EB16; ++b)
#pragma unroll
                for (int kq = 0; kq < 4; ++kq)
                    *reinterpret_cast<uint4 *>(parkB + (b * 4 + kq) * 1024 + lane * 16) = Bst[b][kq].u;
        }

        f32x16 acc[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;

        // running pointer to this lane's first segment of the block being fetched
        const uint16_t *gp = p.gslab + (size_t)q * 8 + 4 * hh + (size_t)(8 * sh) * p.seg_stride;
        int seg0 = 8 * sh;
        uint2 Rg[8];
        auto load_grads = [&]() {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if (ok && seg0 + i < p.S)
                    Rg[i] = *reinterpret_cast<const uint2 *>(gp + (size_t)i * p.seg_stride);
                else
                    Rg[i] = make_uint2(0, 0);
            }
            gp += (size_t)16 * p.seg_stride;
            seg0 += 16;
        };
        load_grads();

#pragma unroll
        for (int kb = 0; kb < KBM; ++kb) {
            if (kb < KB) {
                Frag P[4];
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    *reinterpret_cast<uint2 *>(park + (8 * sh + i) * kDotPitch + c * 16 + hh * 8) = Rg[i];
                // P[j]: element 4hh + j of the chunk, segments 8sh .. 8sh+7 packed as 8 bf16
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int ip = 0; ip < 4; ++ip) {
                        const uint32_t a = (j >> 1) ? Rg[2 * ip].y : Rg[2 * ip].x;
                        const uint32_t b = (j >> 1) ? Rg[2 * ip + 1].y : Rg[2 * ip + 1].x;
                        P[j].w[ip] = (j & 1) ? __builtin_amdgcn_perm(b, a, 0x07060302u)
                                             : __builtin_amdgcn_perm(b, a, 0x05040100u);
                    }
                if (kb + 1 < KB) load_grads();  // next 16 segments, in flight behind the MFMAs
                Frag whi, wlo;
                whi.u = wtab[(kb * 2 + 0) * 64 + lane];
                wlo.u = wtab[(kb * 2 + 1) * 64 + lane];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(whi.v, P[j].v, acc[j], 0, 0, 0);
                    acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wlo.v, P[j].v, acc[j], 0, 0, 0);
                }
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int kq = 0; kq < 4; ++kq) {
                    Frag af;
                    af.u = *reinterpret_cast<const uint4 *>(park + (lane & 15) * kDotPitch +
                                                            (4 * kq + (lane >> 4)) * 16);
#pragma unroll
                    for (int b = 0; b < EB16; ++b) {
                        Frag bf = Bst[b][kq];
                        if constexpr (kParkB)
                            bf.u = *reinterpret_cast<const uint4 *>(parkB + (b * 4 + kq) * 1024 + lane * 16);
                        dots[kb][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af.v, bf.v, dots[kb][b], 0, 0, 0);
                    }
                }
                __builtin_amdgcn_wave_barrier();
            }
        }

        // accumulator element r of lane (c, hh, sh): expert 8*(r>>2) + 4*sh + (r&3), elements 4hh..4hh+3 of chunk c
        if (ok) {
            const long off = rect_offset(p.rc, q) + 4 * hh;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int e = 8 * (r >> 2) + 4 * sh + (r & 3);
                if (e >= Ewin) continue;
                float v[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) v[j] = acc[j][r];
                const size_t eoff = (size_t)(p.e0 + e) * p.rc.expert_stride + off;
                if (p.grad_f32) {
                    float4 *dst = reinterpret_cast<float4 *>(reinterpret_cast<float *>(p.dW) + eoff);
                    float4 o = make_float4(v[0], v[1], v[2], v[3]);
                    if (p.accumulate) {
                        const float4 cur = *dst;
                        o.x += cur.x; o.y += cur.y; o.z += cur.z; o.w += cur.w;
                    }
                    *dst = o;
                } else {
                    uint2 *dst = reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(p.dW) + eoff);
                    if (p.accumulate) {
                        const uint2 cur = *dst;
                        v[0] += __uint_as_float(cur.x << 16);
                        v[1] += __uint_as_float(cur.x & 0xffff0000u);
                        v[2] += __uint_as_float(cur.y << 16);
                        v[3] += __uint_as_float(cur.y & 0xffff0000u);
                    }
                    typedef uint32_t u32x2v __attribute__((ext_vector_type(2)));
                    u32x2v ov;
                    ov.x = pack_bf16(v[0], v[1]);
                    ov.y = pack_bf16(v[2], v[3]);
                    __builtin_nontemporal_store(ov, reinterpret_cast<u32x2v *>(dst));
                }
            }
        }
    }

    // Partial sums of dw per workgroup: the four waves' accumulators are added in wave order in
    // LDS (which nobody needs any more), a later kernel adds the workgroups' slots in slot order.
    // 16x16 accumulator element r: row (segment) 4*(lane>>4) + r, column (expert) lane & 15.
    constexpr int kPer = KBM * EB16 * 4 * 64;  // accumulator values of one wave
    float *red = reinterpret_cast<float *>(smem);
    __syncthreads();
#pragma unroll
    for (int kb = 0; kb < KBM; ++kb)
#pragma unroll
        for (int b = 0; b < EB16; ++b)
#pragma unroll
            for (int r = 0; r < 4; ++r) red[wave * kPer + ((kb * EB16 + b) * 4 + r) * 64 + lane] = dots[kb][b][r];
    __syncthreads();
    float *part = p.partials + (size_t)blockIdx.x * (KBM * 16) * p.pcols;
    for (int idx = tid; idx < kPer; idx += 256) {
        const float v = ((red[idx] + red[kPer + idx]) + red[2 * kPer + idx]) + red[3 * kPer + idx];
        const int l = idx & 63, r = (idx >> 6) & 3, kbb = idx >> 8;
        const int kb = kbb / EB16, b = kbb - kb * EB16;
        const int seg = kb * 16 + 4 * (l >> 4) + r;
        const int e = p.e0 + b * 16 + (l & 15);
        if (e < p.pcols) {
            float *dst = part + (size_t)seg * p.pcols + e;
            *dst = p.partials_add ? (*dst + v) : v;
        }
    }
}

}  // namespace ms
}  // namespace lory
