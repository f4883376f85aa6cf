// Second-generation batched bf16 MFMA GEMM for gfx950: 256 x 256 tiles fed by
// a four-stage LDS ring that is filled with direct global->LDS loads
// (global_load_lds_dwordx4), so that three K steps of operands are in flight
// while one is being multiplied.  Same problem statement, operand layouts and
// epilogue interface as gemm_bf16.h (the dense contractions of the merged FFN,
// paper Section 3.1 / Appendix B); this variant needs M % 256 == 0 and
// N % (256 / NSET) == 0 and is used whenever the shape allows.
//
// Per K step (BK = 32) a stage holds A (16 KB) and B (16 KB).  A direct load
// writes the 64 lanes' 16-byte chunks to 1 KB of consecutive LDS, so the
// swizzles below are applied on the global side: each lane fetches the chunk
// that belongs at its LDS position.
//   K-contiguous operand: rows of 32 bf16 = 4 chunks; chunk c of row r lives in
//     slot c ^ f(r), f(r) = ((r>>1 ^ r>>3) & 1) | ((r>>2 & 1) << 1).
//   operand stored with K as the slow index (read with ds_read_b64_tr_b16):
//     32 K rows of W bf16, dense; the 64-byte granule g of row k lives at
//     granule g ^ (k & 3).
#pragma once

#include "gemm_bf16.h"

namespace lory {
namespace gemm2 {

using gemm::bf16x8;
using gemm::f32x16;
using gemm::Params;
using gemm::s16x4;
using gemm::u32x2;
using gemm::u32x4;

constexpr int kThreads = 256;
constexpr int BM = 256;
constexpr int BK = 32;
constexpr int kStages = 4;
constexpr int kOperandBytes = 16 * 1024;        // one operand of one stage
constexpr int kStageBytes = 2 * kOperandBytes;  // A + B

template <int NSET>
struct Smem {
    static constexpr int BN = 256;  // columns of the tile over all operand sets
    static constexpr int BNS = BN / NSET;
    static constexpr int ring = kStages * kStageBytes;
    static constexpr int out_pitch = BNS * 2 + 16;
    static constexpr int out_bytes = BM * out_pitch;
    static constexpr int total = ring > out_bytes ? ring : out_bytes;
};

__device__ __forceinline__ int fkc(int row)
{
    return (((row >> 1) ^ (row >> 3)) & 1) | (((row >> 2) & 1) << 1);
}

// Element offset (relative to the operand's base pointer at K step 0) of the chunk that belongs
// at LDS chunk position L of a K-contiguous tile.
__device__ __forceinline__ long chunk_off_kc(int L, int ld, int row0)
{
    const int row = L >> 2, slot = L & 3;
    return (long)(row0 + row) * ld + ((slot ^ fkc(row)) << 3);
}

// Same for a tile stored with K as the slow index, W columns wide.
template <int W>
__device__ __forceinline__ long chunk_off_tr(int L, int ld, int col0)
{
    constexpr int cpr = W / 8;
    const int k = L / cpr, pchunk = L % cpr;
    const int g = (pchunk >> 2) ^ (k & 3);
    return (long)k * ld + col0 + (((g << 2) | (pchunk & 3)) << 3);
}

__device__ __forceinline__ bf16x8 frag_kc(const char *lds, int row0, int kk, int lane)
{
    const int row = row0 + (lane & 31);
    const int c = kk * 2 + (lane >> 5);
    return *reinterpret_cast<const bf16x8 *>(lds + row * 64 + ((c ^ fkc(row)) << 4));
}

template <int W>
__device__ __forceinline__ bf16x8 frag_tr(const char *lds, int col0, int kk, int lane)
{
    typedef __attribute__((address_space(3))) s16x4 *lds_ptr;
    const int g16 = lane >> 4, r = lane & 15;
    const int coloff = (col0 + 16 * (g16 & 1) + 4 * (r & 3)) * 2;
    const int krow = kk * 16 + 8 * (g16 >> 1) + (r >> 2);
    const char *p = lds + krow * (W * 2) + ((((coloff >> 6) ^ (krow & 3)) << 6) | (coloff & 63));
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + 4 * W * 2));
    union {
        s16x4 h[2];
        bf16x8 v;
    } u;
    u.h[0] = lo;
    u.h[1] = hi;
    return u.v;
}

// One direct global->LDS load: every lane supplies its own global address, the 64 lanes'
// 16-byte chunks land at lds_addr + 16 * lane (lds_addr is wave-uniform and travels in M0).
// Issued as inline assembly so that the compiler's wait-count bookkeeping does not see an LDS
// writer: completion is tracked by hand with vmcnt below (VMEM operations of a wave retire in
// order), which is what lets three K steps stay in flight across barriers.
__device__ __forceinline__ void dma16(const uint16_t *g, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :
                 : "s"(lds_addr), "v"(g)
                 : "memory", "m0");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Workgroup barrier without the release/acquire fence of __syncthreads() (which would wait for
// every outstanding load): LDS reads of this wave have returned (lgkmcnt) before it arrives.
__device__ __forceinline__ void ring_barrier()
{
    // s_waitcnt lgkmcnt(0) as a builtin (simm16 0xC07F: vmcnt and expcnt left at their maxima) so
    // that the compiler's own LDS bookkeeping knows the reads have returned.
    __builtin_amdgcn_s_waitcnt(0xC07F);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

template <int NSET, int NSRC, bool A_MC, bool B_NC, class Epi>
__global__ __launch_bounds__(kThreads, 1) void gemm2_kernel(const Params p, const Epi epi)
{
    static_assert(NSET == 1 || NSRC == 1, "either two operand sets or two sources");
    using SM = Smem<NSET>;
    constexpr int BNS = SM::BNS;          // columns per operand set
    constexpr int WN = BNS / 2;           // columns per wave and set
    constexpr int MI = 4, NI = WN / 32;   // 128 x WN per wave and set
    constexpr int BSET_BYTES = kOperandBytes / NSET;

    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm0 = (wave >> 1) * 128;
    const int wn0 = (wave & 1) * WN;
    const uint32_t wave_u = __builtin_amdgcn_readfirstlane(wave);
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)smem;

    // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  Give every XCD a
    // contiguous range of tiles so that the tiles of one segment, which share the A operand,
    // meet in the same L2.
    const int tiles_n = p.N / BNS;
    const int tiles_m = p.M / BM;
    const int ntiles = p.batches * tiles_m * tiles_n;
    const int per_xcd = (ntiles + 7) >> 3;
    int bid = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (bid >= ntiles) return;
    const int nt = bid % tiles_n;
    bid /= tiles_n;
    const int mt = bid % tiles_m;
    const int batch = bid / tiles_m;
    const int m0 = mt * BM, n0 = nt * BNS;

    const int ktiles = p.K / BK;
    const int total = ktiles * NSRC;

    // per-lane element offsets of this wave's 4 + 4 chunks per stage
    long offA[4], offB[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int L = (wave * 4 + i) * 64 + lane;  // LDS chunk position inside a 16 KB operand tile
        offA[i] = A_MC ? chunk_off_tr<BM>(L, p.lda[0], m0) : chunk_off_kc(L, p.lda[0], m0);
        const int set = (NSET == 2) ? (L >> 9) : 0;
        const int Ls = (NSET == 2) ? (L & 511) : L;
        (void)set;
        offB[i] = B_NC ? chunk_off_tr<BNS>(Ls, p.ldb[0], n0) : chunk_off_kc(Ls, p.ldb[0], n0);
    }
    const long kstepA = A_MC ? (long)BK * p.lda[0] : BK;
    const long kstepB = B_NC ? (long)BK * p.ldb[0] : BK;

    // One of the 8 direct loads this wave contributes to K step t: i < 4 -> A chunk i, else B chunk i - 4.
    auto issue_one = [&](int t, int i) {
        const int src = (NSRC == 2) ? (t / ktiles) : 0;
        const int ks = t % ktiles;
        const uint32_t stage = lds0 + (t & (kStages - 1)) * kStageBytes + wave_u * 4096;
        if (i < 4) {
            const uint16_t *a = p.A[src] + (size_t)batch * p.a_batch[src] + ks * kstepA;
            dma16(a + offA[i], stage + i * 1024);
        } else {
            const int j = i - 4;
            const int set = (NSET == 2) ? ((wave * 4 + j) >> 3) : 0;  // 8 KB = 8 wave-loads per set
            const int bi = (NSRC == 2) ? src : set;
            const uint16_t *b = p.B[bi] + (size_t)batch * p.b_batch[bi] + ks * kstepB;
            dma16(b + offB[j], stage + kOperandBytes + j * 1024);
        }
    };

    f32x16 acc[NSET][MI][NI];
#pragma unroll
    for (int s = 0; s < NSET; ++s)
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[s][i][j][r] = 0.f;

#pragma unroll
    for (int t = 0; t < kStages - 1; ++t)
        if (t < total) {
#pragma unroll
            for (int i = 0; i < 8; ++i) issue_one(t, i);
        }

    // Fragment f of a 16-wide K slice: f < 4 -> A rows block f, else B columns block f - 4
    // (blocks of B count through the operand sets).
    auto load_frag = [&](const char *la, int kk, int f, bf16x8 (&af)[MI], bf16x8 (&bfr)[NSET * NI]) {
        if (f < 4) {
            if constexpr (A_MC)
                af[f] = frag_tr<BM>(la, wm0 + f * 32, kk, lane);
            else
                af[f] = frag_kc(la, wm0 + f * 32, kk, lane);
        } else {
            const int q = f - 4, s = q / NI, j = q % NI;
            const char *lb = la + kOperandBytes + s * BSET_BYTES;
            if constexpr (B_NC)
                bfr[q] = frag_tr<BNS>(lb, wn0 + j * 32, kk, lane);
            else
                bfr[q] = frag_kc(lb, wn0 + j * 32, kk, lane);
        }
    };
    static_assert(NSET * NI == 4, "a wave multiplies 4 A blocks with 4 B blocks per K slice");

    // The 16 MFMAs of a K slice are issued one per "slot"; every slot also carries one LDS
    // fragment read for the next slice or one direct load for the ring, so that those issue
    // in the shadow of the matrix pipe instead of between bursts.  Fragments are double
    // buffered in registers.  The single barrier of an iteration sits between the two slices
    // of K step t: by then every wave has finished reading step t-1 (its ring slot may be
    // refilled with step t+3) and step t+1 has landed for everyone (its first slice can be
    // fetched behind the second slice's MFMAs).
    bf16x8 a0[MI], b0[NSET * NI], a1[MI], b1[NSET * NI];
    wait_vmcnt<(kStages - 2) * 8>();  // steps 1 and 2 may still be in flight
    if (total < kStages - 1) wait_vmcnt<0>();
    ring_barrier();
#pragma unroll
    for (int f = 0; f < 8; ++f) load_frag(smem, 0, f, a0, b0);

    // REFILL: a K step t+3 exists and is requested now; MORE: a K step t+1 exists.
    auto step = [&](int t, auto refill_c, auto more_c) {
        constexpr bool REFILL = decltype(refill_c)::value;
        constexpr bool MORE = decltype(more_c)::value;
        const char *la = smem + (t & (kStages - 1)) * kStageBytes;
        const char *ln = smem + ((t + 1) & (kStages - 1)) * kStageBytes;
#pragma unroll
        for (int sl = 0; sl < 16; ++sl) {
            const int i = sl >> 2, q = sl & 3;
            acc[q / NI][i][q % NI] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b0[q], a0[i], acc[q / NI][i][q % NI], 0, 0, 0);
            if ((sl & 1) == 0) load_frag(la, 1, sl >> 1, a1, b1);
            __builtin_amdgcn_sched_barrier(0);
        }
        // step t+1 complete for this wave: at most step t+2 pending
        if constexpr (REFILL)
            wait_vmcnt<8>();  // REFILL implies that step t+2 exists
        else
            wait_vmcnt<0>();
        ring_barrier();
#pragma unroll
        for (int sl = 0; sl < 16; ++sl) {
            const int i = sl >> 2, q = sl & 3;
            acc[q / NI][i][q % NI] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b1[q], a1[i], acc[q / NI][i][q % NI], 0, 0, 0);
            if ((sl & 1) == 0) {
                if constexpr (MORE) load_frag(ln, 0, sl >> 1, a0, b0);
            } else {
                if constexpr (REFILL) issue_one(t + kStages - 1, sl >> 1);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    using std::false_type;
    using std::true_type;
    int t = 0;
    for (; t + kStages - 1 < total; ++t) step(t, true_type(), true_type());
    for (; t + 1 < total; ++t) step(t, false_type(), true_type());
    if (t < total) step(t, false_type(), false_type());
    __syncthreads();  // the ring is idle: reuse it as the output staging tile

    typename Epi::In in[MI][NI][4];
    if constexpr (Epi::HAS_IN) {
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int rq = 0; rq < 4; ++rq) {
                    const int m = m0 + wm0 + i * 32 + (lane & 31);
                    const int n = n0 + wn0 + j * 32 + 8 * rq + 4 * (lane >> 5);
                    in[i][j][rq] = epi.load(batch, m, n);
                }
    }
#pragma unroll
    for (int o = 0; o < Epi::NOUT; ++o) {
        if (!epi.enabled(o)) continue;
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int rq = 0; rq < 4; ++rq) {
                    const int ml = wm0 + i * 32 + (lane & 31);
                    const int nl = wn0 + j * 32 + 8 * rq + 4 * (lane >> 5);
                    float v[NSET][4];
#pragma unroll
                    for (int s = 0; s < NSET; ++s)
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[s][e] = acc[s][i][j][rq * 4 + e];
                    const u32x2 pk = epi.pack(o, batch, m0 + ml, n0 + nl, in[i][j][rq], v);
                    *reinterpret_cast<u32x2 *>(smem + ml * SM::out_pitch + nl * 2) = pk;
                }
        __syncthreads();
        constexpr int cpr = BNS / 8;
#pragma unroll 4
        for (int idx = tid; idx < BM * cpr; idx += kThreads) {
            const int row = idx / cpr, c = idx % cpr;
            const u32x4 val = *reinterpret_cast<const u32x4 *>(smem + row * SM::out_pitch + c * 16);
            *reinterpret_cast<u32x4 *>(epi.ptr(o, batch, m0 + row, n0 + c * 8)) = val;
        }
        __syncthreads();
    }
}

// Shapes this kernel accepts.
template <int NSET, int NSRC>
inline bool fits(const Params &p)
{
    if (p.M % BM != 0 || p.N % (256 / NSET) != 0 || p.K % BK != 0) return false;
    if (NSRC == 2 && (p.lda[0] != p.lda[1] || p.ldb[0] != p.ldb[1])) return false;
    if (NSET == 2 && p.ldb[0] != p.ldb[1]) return false;
    return true;
}

template <int NSET, int NSRC, bool A_MC, bool B_NC, class Epi>
inline hipError_t launch(const Params &p, const Epi &epi, hipStream_t st)
{
    using SM = Smem<NSET>;
    auto kern = gemm2_kernel<NSET, NSRC, A_MC, B_NC, Epi>;
    static bool configured = false;  // per instantiation
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, SM::total);
        if (e != hipSuccess) return e;
        configured = true;
    }
    const long ntiles = (long)p.batches * (p.M / BM) * (p.N / SM::BNS);
    const long blocks = (ntiles + 7) / 8 * 8;  // the kernel re-maps block ids per XCD and drops the excess
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(kThreads), SM::total, st, p, epi);
    return hipGetLastError();
}

}  // namespace gemm2
}  // namespace lory
