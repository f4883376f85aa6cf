// Persistent batched bf16 MFMA GEMM for gfx950: 256 x 256 tiles fed by a
// four-stage LDS ring that is filled with direct global->LDS loads
// (global_load_lds_dwordx4), so that two to three K steps of operands are in
// flight while one is being multiplied.  Same problem statement, operand layouts and
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
    // epilogue staging: every wave owns 32 rows x 128 columns of bf16 (one plane of 128 columns, or
    // the two 64-column planes of a combining epilogue), no padding
    static constexpr int stage_out = 32 * 128 * 2;
    static constexpr int total = ring + 4 * stage_out;
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

// Persistent kernel: the grid is one workgroup per CU (a multiple of 8); every workgroup walks
// its own list of tiles, and the K steps of consecutive tiles form one stream through the
// ring, so the first operands of the next tile are already in flight while the current tile
// is multiplied and written out.
template <int NSET, int NSRC, bool A_MC, bool B_NC, class Epi>
__global__ __launch_bounds__(kThreads, 1) void gemm2_kernel(const Params p, const Epi epi)
{
    static_assert(NSET == 1 || NSRC == 1, "either two operand sets or two sources");
    using SM = Smem<NSET>;
    constexpr int BNS = SM::BNS;          // columns per operand set
    constexpr int WN = BNS / 2;           // columns per wave and set
    constexpr int MI = 4, NI = WN / 32;   // 128 x WN per wave and set
    constexpr int BSET_BYTES = kOperandBytes / NSET;
    static_assert(NSET * NI == 4, "a wave multiplies 4 A blocks with 4 B blocks per K slice");

    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm0 = (wave >> 1) * 128;
    const int wn0 = (wave & 1) * WN;
    const uint32_t wave_u = __builtin_amdgcn_readfirstlane(wave);
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)smem;

    // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  Every XCD gets a
    // contiguous range of tiles, shared cyclically by its workgroups, so that the tiles of one
    // segment, which share the A operand, meet in the same L2.
    const int tiles_n = p.N / BNS;
    const int tiles_m = p.M / BM;
    const int ntiles = p.batches * tiles_m * tiles_n;
    const int per_xcd = (ntiles + 7) >> 3;
    const int wg_per_xcd = gridDim.x >> 3;
    const int xcd = blockIdx.x & 7, qx = blockIdx.x >> 3;
    int xcd_tiles = ntiles - xcd * per_xcd;  // tiles in this XCD's range
    if (xcd_tiles > per_xcd) xcd_tiles = per_xcd;
    const int my_tiles = (xcd_tiles > qx) ? (xcd_tiles - qx + wg_per_xcd - 1) / wg_per_xcd : 0;
    if (my_tiles == 0) return;

    const int ktiles = p.K / BK;
    const int total = ktiles * NSRC;   // K steps per tile
    const int G = my_tiles * total;    // K steps of this workgroup

    // per-lane element offsets of this wave's 4 + 4 chunks per stage, relative to the tile origin
    long offA[4], offB[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int L = (wave * 4 + i) * 64 + lane;  // LDS chunk position inside a 16 KB operand tile
        offA[i] = A_MC ? chunk_off_tr<BM>(L, p.lda[0], 0) : chunk_off_kc(L, p.lda[0], 0);
        const int Ls = (NSET == 2) ? (L & 511) : L;
        offB[i] = B_NC ? chunk_off_tr<BNS>(Ls, p.ldb[0], 0) : chunk_off_kc(Ls, p.ldb[0], 0);
    }
    const long kstepA = A_MC ? (long)BK * p.lda[0] : BK;
    const long kstepB = B_NC ? (long)BK * p.ldb[0] : BK;

    auto tile_coords = [&](int i, int &batch, int &m0, int &n0) {
        int id = xcd * per_xcd + qx + i * wg_per_xcd;
        const int nt = id % tiles_n;
        id /= tiles_n;
        const int mt = id % tiles_m;
        batch = id / tiles_m;
        m0 = mt * BM;
        n0 = nt * BNS;
    };

    // The A and the B operand of a K step are fetched at different times (see step()), so each
    // load stream keeps the origin (in elements) of the tile it is currently in.
    int ldA_tile = -1, ldB_tile = -1;
    long tileA = 0, tileB = 0;
    int ldA_batch = 0, ldB_batch = 0;
    auto enter_tile_A = [&](int i) {
        int m0, n0;
        tile_coords(i, ldA_batch, m0, n0);
        tileA = A_MC ? (long)m0 : (long)m0 * p.lda[0];
        ldA_tile = i;
    };
    auto enter_tile_B = [&](int i) {
        int m0, n0;
        tile_coords(i, ldB_batch, m0, n0);
        tileB = B_NC ? (long)n0 : (long)n0 * p.ldb[0];
        ldB_tile = i;
    };

    // The 4 + 4 direct loads this wave contributes to K step gsrc of its stream (A chunk i, B
    // chunk j); gslot = K step whose ring slot receives them.
    auto issue_A = [&](int gsrc, int gslot, int i) {
        const int t = gsrc % total;
        const int src = (NSRC == 2) ? (t / ktiles) : 0;
        const int ks = t % ktiles;
        const uint32_t stage = lds0 + (gslot & (kStages - 1)) * kStageBytes + wave_u * 4096;
        const uint16_t *a = p.A[src] + (size_t)ldA_batch * p.a_batch[src] + tileA + ks * kstepA;
        dma16(a + offA[i], stage + i * 1024);
    };
    auto issue_B = [&](int gsrc, int gslot, int j) {
        const int t = gsrc % total;
        const int src = (NSRC == 2) ? (t / ktiles) : 0;
        const int ks = t % ktiles;
        const uint32_t stage = lds0 + (gslot & (kStages - 1)) * kStageBytes + wave_u * 4096;
        const int set = (NSET == 2) ? ((wave * 4 + j) >> 3) : 0;  // 8 KB = 8 wave-loads per set
        const int bi = (NSRC == 2) ? src : set;
        const uint16_t *b = p.B[bi] + (size_t)ldB_batch * p.b_batch[bi] + tileB + ks * kstepB;
        dma16(b + offB[j], stage + kOperandBytes + j * 1024);
    };

    f32x16 acc[NSET][MI][NI];
    auto zero_acc = [&]() {
#pragma unroll
        for (int s = 0; s < NSET; ++s)
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[s][i][j][r] = 0.f;
    };

    for (int g = 0; g < kStages; ++g) {  // the whole ring: K steps 0 .. 3
        const int gsrc = g < G ? g : G - 1;
        if (gsrc / total != ldA_tile) enter_tile_A(gsrc / total);
        if (gsrc / total != ldB_tile) enter_tile_B(gsrc / total);
#pragma unroll
        for (int i = 0; i < 4; ++i) issue_A(gsrc, g, i);
#pragma unroll
        for (int j = 0; j < 4; ++j) issue_B(gsrc, g, j);
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

    // The 16 MFMAs of a K slice are issued one per "slot"; every slot also carries one LDS
    // fragment read for the next slice or one direct load for the ring, so that those issue
    // in the shadow of the matrix pipe instead of between bursts.  Fragments are double
    // buffered in registers.  The single barrier of a K step sits between its two slices: by
    // then every wave has finished reading step g-1 (its ring slot may be refilled with step
    // g+3) and step g+1 has landed for everyone (its first slice can be fetched behind the
    // second slice's MFMAs).
    bf16x8 a0[MI], b0[NSET * NI], a1[MI], b1[NSET * NI];
    wait_vmcnt<(kStages - 1) * 8>();  // steps 1 .. 3 may still be in flight
    ring_barrier();
#pragma unroll
    for (int f = 0; f < 8; ++f) load_frag(smem, 0, f, a0, b0);

    // One K step g.  Its 32 MFMA slots also carry the LDS fragment reads of the next slice (even
    // slots) and this wave's eight direct loads for the ring, one every fourth slot, spread over
    // the whole step: the four waves issue theirs at the same time, and the memory pipeline takes
    // about 16 cycles per load, so loads in adjacent slots (as when all eight sat in one half
    // step) stalled the waves for longer than the MFMAs they hide behind.  (Giving every wave
    // slots of its own was tried: the wave-dependent branches cost far more than they saved.)
    //   first half:  A chunks of step g+3 (into the slot step g-1 left at the previous barrier)
    //   second half: B chunks of step g+4 (into the slot step g itself left at this step's
    //                barrier: every wave has fetched its last fragments of step g by then)
    // so that, with the four ring slots, up to three and a half K steps of operands are in
    // flight.  The B operand is the one that streams from HBM, hence the longer lead.  Across a
    // tile boundary the A chunks that the next tile's first step would issue are issued half a
    // step early, in the last step of the tile, so that everything the next tile's first three
    // steps wait for is older than the epilogue's stores: loads and stores share vmcnt and
    // retire in order, and a wait may only leave younger operations pending.
    // Past the end of the stream the loads re-fetch the last K step into slots nobody reads, so
    // "all but the newest 16 loads have landed" (vmcnt(16)) always means "step g+1 is complete".
    // extra_now: store instructions of the previous tile's epilogue that may still be pending
    // (only non-zero for the first three steps of a tile).
    auto step = [&](int g, int extra_now, bool first_of_tile, bool last_of_tile) {
        const char *la = smem + (g & (kStages - 1)) * kStageBytes;
        const char *ln = smem + ((g + 1) & (kStages - 1)) * kStageBytes;
        const int srcA = (g + 3 < G) ? (g + 3) : (G - 1);
        if (!first_of_tile && srcA / total != ldA_tile) enter_tile_A(srcA / total);
#pragma unroll
        for (int sl = 0; sl < 16; ++sl) {
            const int i = sl >> 2, q = sl & 3;
            acc[q / NI][i][q % NI] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b0[q], a0[i], acc[q / NI][i][q % NI], 0, 0, 0);
            if ((sl & 1) == 0) load_frag(la, 1, sl >> 1, a1, b1);
            if (!first_of_tile && (sl & 3) == 1) issue_A(srcA, g + 3, sl >> 2);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (extra_now == 32)
            wait_vmcnt<48>();
        else if (extra_now == 16)
            wait_vmcnt<32>();
        else
            wait_vmcnt<16>();
        ring_barrier();
        const int srcB = (g + 4 < G) ? (g + 4) : (G - 1);  // K step to fetch
        if (srcB / total != ldB_tile) enter_tile_B(srcB / total);
        if (last_of_tile && srcB / total != ldA_tile) enter_tile_A(srcB / total);
#pragma unroll
        for (int sl = 0; sl < 16; ++sl) {
            const int i = sl >> 2, q = sl & 3;
            acc[q / NI][i][q % NI] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b1[q], a1[i], acc[q / NI][i][q % NI], 0, 0, 0);
            if ((sl & 1) == 0) load_frag(ln, 0, sl >> 1, a0, b0);
            if ((sl & 3) == 1) issue_B(srcB, g + 4, sl >> 2);
            if (last_of_tile && (sl & 3) == 3) issue_A(srcB, g + 4, sl >> 2);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // Epilogue of one tile, wave-local: the wave's 128 x WN sub-tile leaves in blocks of 32 rows
    // through the wave's own staging area (XOR-swizzled 16-byte chunks), as 16-byte stores that
    // are contiguous along n.  Accumulator element r of a 32x32 block is row m = lane & 31,
    // column n = 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3).
    char *stg = smem + SM::ring + wave * SM::stage_out;
    constexpr int CP = WN / 8;  // 16-byte chunks per staged row
    auto epilogue = [&](int tile_i) {
        int batch, m0, n0;
        tile_coords(tile_i, batch, m0, n0);
        const int r = lane & 31, h = lane >> 5;
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            if constexpr (Epi::COMBINE) {
                // One output plane computed from both operand sets: both are staged as bf16 and
                // combined on the way out.  (Combined straight from the accumulators, the compiler
                // copied the whole second set to VGPRs at the top of the epilogue and spilled.)
                static_assert(NSET == 2, "a combining epilogue has two operand sets");
                constexpr int PLB = 32 * WN * 2;
#pragma unroll
                for (int s = 0; s < NSET; ++s)
#pragma unroll
                    for (int j = 0; j < NI; ++j)
#pragma unroll
                        for (int rq = 0; rq < 4; ++rq) {
                            const int c = (j * 32 + 8 * rq) >> 3;
                            u32x2 pk;
                            pk.x = gemm::cvt_pk_bf16(acc[s][i][j][rq * 4 + 0], acc[s][i][j][rq * 4 + 1]);
                            pk.y = gemm::cvt_pk_bf16(acc[s][i][j][rq * 4 + 2], acc[s][i][j][rq * 4 + 3]);
                            *reinterpret_cast<u32x2 *>(stg + s * PLB + r * (WN * 2) + ((c ^ (r & (CP - 1))) << 4) + h * 8) = pk;
                            __builtin_amdgcn_sched_barrier(0);
                        }
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int it = 0; it < (32 * CP) / 64; ++it) {
                    const int idx = it * 64 + lane;
                    const int row = idx / CP, c = idx % CP;
                    const int off = row * (WN * 2) + ((c ^ (row & (CP - 1))) << 4);
                    const u32x4 v0 = *reinterpret_cast<const u32x4 *>(stg + off);
                    const u32x4 v1 = *reinterpret_cast<const u32x4 *>(stg + PLB + off);
                    __builtin_nontemporal_store(
                        epi.combine(v0, v1),
                        reinterpret_cast<u32x4 *>(epi.ptr(Epi::COMBINED_PLANE, batch, m0 + wm0 + i * 32 + row, n0 + wn0 + c * 8)));
                }
                __builtin_amdgcn_wave_barrier();
                continue;
            }
            // all planes of one 32-row block before the next block: its accumulators are read
            // into registers once
#pragma unroll
            for (int o = 0; o < Epi::NOUT; ++o) {
                if (!epi.enabled(o)) continue;
#pragma unroll
                for (int j = 0; j < NI; ++j)
#pragma unroll
                    for (int rq = 0; rq < 4; ++rq) {
                        const int nl = j * 32 + 8 * rq + 4 * h;  // column inside the wave's WN columns
                        float v[NSET][4];
#pragma unroll
                        for (int s = 0; s < NSET; ++s)
#pragma unroll
                            for (int e = 0; e < 4; ++e) v[s][e] = acc[s][i][j][rq * 4 + e];
                        const u32x2 pk = epi.pack(o, batch, m0 + wm0 + i * 32 + r, n0 + wn0 + nl, typename Epi::In(), v);
                        const int c = nl >> 3;
                        *reinterpret_cast<u32x2 *>(stg + r * (WN * 2) + ((c ^ (r & (CP - 1))) << 4) + h * 8) = pk;
                        __builtin_amdgcn_sched_barrier(0);  // one quad at a time: keeps register use flat
                    }
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int it = 0; it < (32 * CP) / 64; ++it) {
                    const int idx = it * 64 + lane;
                    const int row = idx / CP, c = idx % CP;
                    const u32x4 val = *reinterpret_cast<const u32x4 *>(stg + row * (WN * 2) + ((c ^ (row & (CP - 1))) << 4));
                    // streamed output: non-temporal, so that it does not push the operands that later
                    // tiles share (activations of the segment) out of the caches
                    __builtin_nontemporal_store(
                        val, reinterpret_cast<u32x4 *>(epi.ptr(o, batch, m0 + wm0 + i * 32 + row, n0 + wn0 + c * 8)));
                }
                __builtin_amdgcn_wave_barrier();
            }
        }
    };

    // 16-byte store instructions a wave issues per tile epilogue
    int nst = 0;
#pragma unroll
    for (int o = 0; o < Epi::NOUT; ++o)
        if (epi.enabled(o)) nst += MI * ((32 * CP) / 64);
    const int extra = (total >= 2) ? (nst >= 32 ? 32 : (nst >= 16 ? 16 : 0)) : 0;
    int g = 0;
    for (int tile_i = 0; tile_i < my_tiles; ++tile_i) {
        zero_acc();
        // the first three K steps of a tile run while the previous tile's stores drain
        const int relaxed = (tile_i > 0) ? 3 : 0;
        for (int t = 0; t < total; ++t, ++g) step(g, t < relaxed ? extra : 0, t == 0, t == total - 1);
        epilogue(tile_i);
    }
    wait_vmcnt<0>();  // no direct load may still be writing LDS when the workgroup retires
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

inline int persistent_grid()
{
    static int grid = 0;
    if (grid == 0) {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 8)
            cus = 256;
        grid = cus / 8 * 8;
    }
    return grid;
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
    long blocks = (ntiles + 7) / 8 * 8;
    if (blocks > persistent_grid()) blocks = persistent_grid();  // one workgroup per CU walks several tiles
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(kThreads), SM::total, st, p, epi);
    return hipGetLastError();
}

}  // namespace gemm2
}  // namespace lory
