// Expert gradients without per-segment weight gradients in memory (paper Section 3.1 / Eq. 2,
// backward of the merge; Appendix B's E/T overhead):
//     dW[e]    = sum_s w[s, e] * (A_s^T B_s)            (adjoint of the merge)
//     dw[s, e] = < W[e], A_s^T B_s >                    (gradient of the routing weights)
// for one expert matrix W [E][M][N], with A [tokens][M] and B [tokens][N] the two token-major
// operands of its weight gradient (X and dG / dU for the gate / up matrices, A and dY for the down
// matrix).  At most 16 experts, bf16 gradients.
//
// A workgroup (4 wavefronts, one per CU) owns a 64 x 64 tile of the matrix for all experts: its
// 16 x 4096 fp32 expert-gradient accumulators are all of the CU's accumulation registers.  It walks
// the token stream once, 64 tokens per step through a five-stage ring of direct global->LDS loads
// shared by the four waves (four steps, 64 KB, in flight: a step has only four MFMAs per wave, so
// the ring has to cover the whole load latency); wave (wm, wn) multiplies its 32 x 32 block.  At the end of a segment the
// block P_s (the segment's weight gradient) is rounded to bf16 and written to LDS as
// P[cell][segment of the group]; after every eighth segment the wave
//   * adds P_s to the expert gradients: 64 MFMAs 16x16x32, rows = experts, columns = 16 cells,
//     K = 8 segments x (hi, lo) of the fp32 routing weights, upper half of K zero (operand: a
//     cell's 16-byte row);
//   * forms < W[e], P_s > for its elements: 32 MFMAs 16x16x32, rows = experts, columns = segments,
//     K = 32 cells (operand: two transposing LDS reads of four cells' rows each); the wave's part of
//     the W tile stays on chip for the whole task, 112 registers and 4 KB of LDS; the sums are added
//     to the wave's own slot of a partial-sum buffer (fixed order: reproducible).
// Everything after the ring is wave-private: no barrier besides the ring's.
//
// LDS (160 KB): ring 5 x 16 KB | P: per wave [1024 cells][8 segments] bf16 | per wave 8 K blocks of
// the W tile ([block][lane] x 8 bytes).
//   cell c = ((r >> 2) * 2 + h) * 128 + (r & 3) * 32 + m       accumulator element r of lane (m, h):
//            row m, column 8 (r >> 2) + 4 h + (r & 3) of the wave's block
//   K block j of the inner products, operand lane (x, kg), element t: cell (j >> 3) * 128 + t * 32 +
//            4 (j & 7) + kg, i.e. row 4 (j & 7) + kg, columns 8 (j >> 4) + 4 ((j >> 3) & 1) + t.
#pragma once

#include "gemm2_bf16.h"
#include "merge_scatter_bf16.h"

namespace lory {
namespace fsg {

using gemm::bf16x8;
using gemm::f32x16;
using gemm::s16x4;
using gemm::u32x2;
using gemm::u32x4;
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int BT = 64;                    // tile edge
constexpr int BK = 64;                    // tokens per step
constexpr int kStages = 5;
constexpr int kOperand = BK * BT * 2;     // 8 KB: 64 token rows of 64 columns
constexpr int kStage = 2 * kOperand;      // A + B
constexpr int kRing = kStages * kStage;   // 80 KB
constexpr int kP = 16 * 1024;             // one wave's P region
constexpr int kWRegs = 56;                // K blocks of the W tile held in registers; the other 8 in LDS
constexpr int kWL = (64 - kWRegs) * 512;  // one wave's part of the W tile in LDS: 4 KB
constexpr int kLds = kRing + 4 * kP + 4 * kWL;   // 160 KB
constexpr int kSegments = 8;              // segments per group step

struct Params {
    const uint16_t *A;      // [tokens][lda]
    const uint16_t *B;      // [tokens][ldb]
    int lda, ldb;
    const uint16_t *W;      // expert e at W + e * expert_stride, row-major [M][ldw]
    uint16_t *dW;           // same addressing as W
    long expert_stride;
    int ldw;
    const float *w;         // [S][E]
    int E, T, S, M, N;
    float *partials;        // [gridDim.x * 4][S][16]
    int partials_add;       // add to what the buffer holds instead of overwriting it
};

// One K-slow operand fragment of a 32 x 32 x 16 MFMA: columns col0 .. col0 + 31 of the 64-column
// tile, K rows 16 kk .. 16 kk + 15.  Rows are 128 bytes; the 64-byte half g of row k lives at half
// g ^ ((k >> 1) & 1).
__device__ __forceinline__ bf16x8 frag_tr64(const char *lds, int col0, int kk, int lane)
{
    typedef __attribute__((address_space(3))) s16x4 *lds_ptr;
    const int g16 = lane >> 4, r = lane & 15;
    const int coloff = (col0 + 16 * (g16 & 1) + 4 * (r & 3)) * 2;
    const int krow = kk * 16 + 8 * (g16 >> 1) + (r >> 2);
    const char *p = lds + krow * 128 + ((((coloff >> 6) ^ ((krow >> 1) & 1)) << 6) | (coloff & 63));
    union {
        s16x4 h[2];
        bf16x8 v;
    } u;
    u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
    u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + 4 * 128));
    return u.v;
}

template <int kSegGroup>   // segments per group step: 8
__global__ __launch_bounds__(kThreads, 1) void fsg_kernel(const Params p)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const uint32_t wave_u = __builtin_amdgcn_readfirstlane(wave);
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)smem;
    char *P1 = smem + kRing + wave * kP;
    char *WL = smem + kRing + 4 * kP + wave * kWL;
    float *slot = p.partials + ((size_t)blockIdx.x * 4 + wave) * (size_t)p.S * 16;

    const int ml = lane & 31, h = lane >> 5;      // accumulator lane of the 32 x 32 block
    const int x = lane & 15, kg = lane >> 4;      // operand lane of the 16 x 16 x 16 MFMAs
    const int G = (p.S * p.T) / BK;               // K steps of a task
    const int steps_per_seg = p.T / BK;

    const int tiles_m = p.M / BT, tiles_n = p.N / BT;
    const int mg = (tiles_m + 7) >> 3, ng = (tiles_n + 3) >> 2;
    const int nsuper = mg * ng;
    const int xcd = blockIdx.x & 7, q0 = blockIdx.x >> 3, wg_per_xcd = gridDim.x >> 3;

    // this wave's four direct loads per step: chunks 256 w .. 256 w + 255 of the stage's 1024
    // (waves 0, 1: the A tile, waves 2, 3: the B tile); chunk L of an operand is token row L / 8,
    // 16-byte piece L % 8
    int ld_row[4], ld_col[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int L = ((wave & 1) * 4 + i) * 64 + lane;
        const int k = L >> 3, pc = L & 7;
        const int g = (pc >> 2) ^ ((k >> 1) & 1);
        ld_row[i] = k;
        ld_col[i] = ((g << 2) | (pc & 3)) << 3;
    }
    const bool loads_a = wave < 2;

    bool visited = false;   // this workgroup has run a task (its partial sums hold this launch's values)
    for (int sup = xcd; sup < nsuper; sup += 8) {
        for (int q = q0; q < 32; q += wg_per_xcd) {
            const int mt = (sup % mg) * 8 + (q & 7);
            const int nt = (sup / mg) * 4 + (q >> 3);
            if (mt >= tiles_m || nt >= tiles_n) continue;   // uniform over the workgroup
            const int m0 = mt * BT, n0 = nt * BT;
            const bool add_partials = p.partials_add || visited;
            visited = true;

            // ---- the wave's part of the expert tile, as operands of the inner-product MFMAs:
            //      K block j, lane (e = x, kg): elements 16 j + 4 kg .. + 3, i.e. row 4 (j & 7) + kg,
            //      columns 8 (j >> 4) + 4 ((j >> 3) & 1) .. + 3 of the wave's 32 x 32 block
            u32x2 Wreg[kWRegs];
            {
                const int e = x < p.E ? x : 0;
                const uint16_t *wb = p.W + (size_t)e * p.expert_stride + (size_t)(m0 + wm * 32) * p.ldw + n0 + wn * 32;
#pragma unroll
                for (int j = 0; j < 64; ++j) {
                    const int row = 4 * (j & 7) + kg, col = 8 * (j >> 4) + 4 * ((j >> 3) & 1);
                    u32x2 v = *reinterpret_cast<const u32x2 *>(wb + (size_t)row * p.ldw + col);
                    if (x >= p.E) v = u32x2{0u, 0u};
                    if (j < kWRegs)
                        Wreg[j] = v;
                    else
                        *reinterpret_cast<u32x2 *>(WL + (j - kWRegs) * 512 + lane * 8) = v;
                }
            }

            f32x4 acc_dw[64];   // block b: experts 4 (lane >> 4) .. + 3 (registers) x cell 16 b + (lane & 15)
#pragma unroll
            for (int b = 0; b < 64; ++b) acc_dw[b] = f32x4{0.f, 0.f, 0.f, 0.f};
            f32x16 acc_p;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc_p[r] = 0.f;
            uint32_t even[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};   // an even segment's block as bf16 pairs

            const uint16_t *src = loads_a ? p.A + m0 : p.B + n0;
            const int ld = loads_a ? p.lda : p.ldb;
            auto issue = [&](int g, int stage) {
                const uint32_t dst = lds0 + stage * kStage + wave_u * 4096;
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    gemm2::dma16(src + (size_t)(g * BK + ld_row[i]) * ld + ld_col[i], dst + i * 1024);
            };

            // ring: four steps ahead
#pragma unroll
            for (int i = 0; i < kStages - 1; ++i)
                if (i < G) issue(i, i);
            int g = 0, stage = 0;   // step, its ring stage (g mod 5)
            for (int s0 = 0; s0 < p.S; s0 += kSegGroup) {
                for (int sl = 0; sl < kSegGroup; ++sl) {
                    for (int ks = 0; ks < steps_per_seg; ++ks, ++g) {
                        // own loads of step g have landed (four per step; up to three later steps pending)
                        const int later = G - 1 - g;
                        if (later >= 3)
                            gemm2::wait_vmcnt<12>();
                        else if (later == 2)
                            gemm2::wait_vmcnt<8>();
                        else if (later == 1)
                            gemm2::wait_vmcnt<4>();
                        else
                            gemm2::wait_vmcnt<0>();
                        gemm2::ring_barrier();   // everyone's loads of step g landed; nobody reads step g - 1 any more
                        if (g + kStages - 1 < G) issue(g + kStages - 1, stage == 0 ? kStages - 1 : stage - 1);

                        const char *la = smem + stage * kStage;
                        const char *lb = la + kOperand;
                        stage = (stage == kStages - 1) ? 0 : stage + 1;
#pragma unroll
                        for (int kk = 0; kk < 4; ++kk) {
                            const bf16x8 af = frag_tr64(la, wm * 32, kk, lane);
                            const bf16x8 bfr = frag_tr64(lb, wn * 32, kk, lane);
                            acc_p = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr, af, acc_p, 0, 0, 0);
                        }
                    }
                    // ---- end of segment s0 + sl: acc_p element r = row ml, column 8 (r >> 2) + 4 h + (r & 3).
                    //      An even segment waits in registers for the odd one: 4-byte stores of a segment
                    //      pair (the cells are 16 bytes apart, four lanes share a bank).
#pragma unroll
                    for (int rq = 0; rq < 4; ++rq) {
                        const uint32_t lo = gemm::cvt_pk_bf16(acc_p[rq * 4 + 0], acc_p[rq * 4 + 1]);
                        const uint32_t hi = gemm::cvt_pk_bf16(acc_p[rq * 4 + 2], acc_p[rq * 4 + 3]);
                        if ((sl & 1) == 0) {
                            even[rq * 2 + 0] = lo;
                            even[rq * 2 + 1] = hi;
                        } else {
                            const int cb = (rq * 2 + h) * 128;
                            // P[cell][segment]: segments sl - 1 (low half) and sl
                            uint32_t *p1 = reinterpret_cast<uint32_t *>(P1) + (sl >> 1);
                            const uint32_t el = even[rq * 2 + 0], eh = even[rq * 2 + 1];
                            p1[(cb + 0 * 32 + ml) * 4] = __builtin_amdgcn_perm(lo, el, 0x05040100u);
                            p1[(cb + 1 * 32 + ml) * 4] = __builtin_amdgcn_perm(lo, el, 0x07060302u);
                            p1[(cb + 2 * 32 + ml) * 4] = __builtin_amdgcn_perm(hi, eh, 0x05040100u);
                            p1[(cb + 3 * 32 + ml) * 4] = __builtin_amdgcn_perm(hi, eh, 0x07060302u);
                        }
                    }
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc_p[r] = 0.f;
                }

                // ---- group of eight segments s0 .. s0 + 7
                gemm::bf16x8 wfrag;   // K index 8 kg + i: segment i, hi (kg = 0) or lo (kg = 1) part; zero above
                {
                    union {
                        uint32_t w[4];
                        gemm::bf16x8 v;
                    } u;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        float part[2];
#pragma unroll
                        for (int t = 0; t < 2; ++t) {
                            const float v = (x < p.E && kg < 2) ? p.w[(size_t)(s0 + 2 * i + t) * p.E + x] : 0.f;
                            const float hi = gemm::bf16_bits_to_float(gemm::float_to_bf16_bits(v));
                            part[t] = (kg == 0) ? hi : v - hi;
                        }
                        u.w[i] = gemm::cvt_pk_bf16(part[0], part[1]);
                    }
                    wfrag = u.v;
                }
#pragma unroll
                for (int b = 0; b < 64; ++b) {
                    // every lane supplies its cell's eight segments; the K groups 2 and 3 meet zeros
                    const gemm::bf16x8 pb = *reinterpret_cast<const gemm::bf16x8 *>(P1 + (16 * b + x) * 16);
                    acc_dw[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wfrag, pb, acc_dw[b], 0, 0, 0);
                    if ((b & 3) == 3) __builtin_amdgcn_sched_barrier(0);   // a few reads ahead, not all 64
                }
                f32x4 dots = f32x4{0.f, 0.f, 0.f, 0.f};   // experts 4 kg .. + 3 x segment x & 7
                {
                    // transposing read: within a group of 16 lanes, lane x reads 8 bytes (segments
                    // 4 (x & 1) .. + 3 of cell t = x >> 2 of the K block) and receives, as element t,
                    // what lane 4 t + (x >> 2) read at position x & 3: segment x & 7 of cell t
                    typedef __attribute__((address_space(3))) s16x4 *lds_ptr;
                    const char *pt = P1 + ((x >> 2) * 32 + kg) * 16 + (x & 1) * 8;
#pragma unroll
                    for (int jj = 0; jj < 32; ++jj) {
                        union {
                            u32x2 u[2];
                            s16x4 h[2];
                            gemm::bf16x8 v;
                        } wj, pj;
#pragma unroll
                        for (int u = 0; u < 2; ++u) {
                            const int j = 2 * jj + u;
                            if (j < kWRegs)
                                wj.u[u] = Wreg[j];
                            else
                                wj.u[u] = *reinterpret_cast<const u32x2 *>(WL + (j - kWRegs) * 512 + lane * 8);
                            pj.h[u] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                                (lds_ptr)(pt + ((j >> 3) * 128 + 4 * (j & 7)) * 16));
                        }
                        dots = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wj.v, pj.v, dots, 0, 0, 0);
                        if ((jj & 3) == 3) __builtin_amdgcn_sched_barrier(0);
                    }
                }
                if (x < kSegGroup) {
                    f32x4 *dst = reinterpret_cast<f32x4 *>(slot + (size_t)(s0 + x) * 16 + 4 * kg);
                    f32x4 v = dots;
                    if (add_partials) {
                        const f32x4 old = *dst;
                        v = f32x4{old[0] + dots[0], old[1] + dots[1], old[2] + dots[2], old[3] + dots[3]};
                    }
                    *dst = v;
                }
            }

            // ---- expert gradients out, wave-local through the wave's P1 region: rows 16 mh .. + 15 of
            //      the block at a time as [expert][row][32 columns] bf16 (16 KB)
            __builtin_amdgcn_s_waitcnt(0xC07F);
#pragma unroll
            for (int mh = 0; mh < 2; ++mh) {
#pragma unroll
                for (int rq = 0; rq < 4; ++rq)
#pragma unroll
                    for (int hh = 0; hh < 2; ++hh)
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            // blocks b = ((rq * 2 + hh) * 4 + c4) * 2 + mh hold columns 8 rq + 4 hh + c4
                            u32x2 v;
                            v.x = gemm::cvt_pk_bf16(acc_dw[((rq * 2 + hh) * 4 + 0) * 2 + mh][t],
                                                    acc_dw[((rq * 2 + hh) * 4 + 1) * 2 + mh][t]);
                            v.y = gemm::cvt_pk_bf16(acc_dw[((rq * 2 + hh) * 4 + 2) * 2 + mh][t],
                                                    acc_dw[((rq * 2 + hh) * 4 + 3) * 2 + mh][t]);
                            *reinterpret_cast<u32x2 *>(P1 + ((4 * kg + t) * 16 + x) * 64 + (8 * rq + 4 * hh) * 2) = v;
                            __builtin_amdgcn_sched_barrier(0);
                        }
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int it = 0; it < 16; ++it) {
                    const int qd = it * 64 + lane;            // 16-byte piece of the staged 16 KB
                    const int e = qd >> 6, row = (qd >> 2) & 15, c = qd & 3;
                    const u32x4 val = *reinterpret_cast<const u32x4 *>(P1 + qd * 16);
                    if (e < p.E)
                        *reinterpret_cast<u32x4 *>(p.dW + (size_t)e * p.expert_stride +
                                                   (size_t)(m0 + wm * 32 + mh * 16 + row) * p.ldw + n0 + wn * 32 + c * 8) = val;
                }
                __builtin_amdgcn_wave_barrier();
            }
            __builtin_amdgcn_s_waitcnt(0xC07F);
            gemm2::ring_barrier();   // the next task refills the ring and P1
        }
    }
    if (!visited && !p.partials_add) {
        // a workgroup without a task still owns partial-sum slots: they must read as zero
        for (int i = lane; i < p.S * 16; i += 64) slot[i] = 0.f;
    }
    gemm2::wait_vmcnt<0>();
}

inline bool fits(const Params &p)
{
    return p.E >= 1 && p.E <= 16 && p.M % BT == 0 && p.N % BT == 0 && p.T % BK == 0 &&
           p.S % kSegments == 0 && p.ldw % 8 == 0 && p.lda % 8 == 0 && p.ldb % 8 == 0;
}

inline int grid_size(const Params &p)
{
    const long tasks = (long)(p.M / BT) * (p.N / BT);
    long blocks = (tasks + 7) / 8 * 8;
    if (blocks > gemm2::persistent_grid()) blocks = gemm2::persistent_grid();
    return (int)blocks;
}

inline hipError_t launch(const Params &p, hipStream_t st)
{
    static bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(fsg_kernel<kSegments>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
        if (e != hipSuccess) return e;
        configured = true;
    }
    hipLaunchKernelGGL(fsg_kernel<kSegments>, dim3((unsigned)grid_size(p)), dim3(kThreads), kLds, st, p);
    return hipGetLastError();
}

}  // namespace fsg
}  // namespace lory
