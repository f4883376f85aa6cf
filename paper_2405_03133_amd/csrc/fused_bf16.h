// Merge inside the GEMM: the segment's merged expert matrix (paper Eq. 2,
// theta_bar = sum_e w[s,e] theta_e) is formed tile by tile on chip and fed
// straight to the token contraction of Section 3.1 / Appendix B, so that no
// merged parameter ever reaches HBM.  gfx950, bf16 operands, fp32 accumulation.
//
//     C[t, n] = sum over sources q, k of  A_q[t, k] * Wbar_q(seg(t))[k, n],
//     Wbar_q(s) = sum_e w[s, e] W_q[e]
//
// A workgroup (4 wavefronts) owns a task: R = 4 * WROWS consecutive token rows
// (SC = R / T whole segments) times 64 output columns, with all 65536 (WROWS =
// 256) fp32 accumulators of the CU.  Per 16-wide K slice
//   * every wavefront merges a quarter of the slice's 16 x 64 expert elements for
//     all SC segments with v_mfma_f32_16x16x32_bf16 (rows = segments, K = experts,
//     routing weights as bf16 hi + lo pairs, expert chunks transposed in registers
//     as in the stand-alone merge kernel) and writes the bf16 result to LDS;
//   * after one barrier every wavefront multiplies its own rows (token tiles
//     arrive through a wave-private ring of direct global->LDS loads) with the
//     merged tile of the segment the rows belong to.
// Bytes entering the CU per K slice of 16: 2 * 16 * (E * 64 + R) against
// 2 * 16 * 64 * R flops, i.e. 21 flop/byte at E = 32, R = 1024 (32 at E = 16):
// the kernel is bound by the L2 -> CU path, not by HBM.  It does not depend on
// the segment length except through SC, which is what makes it the better
// choice for short segments, where the slab pipeline (merge kernel + batched
// GEMM) moves S * d * d_ff merged values through HBM for only T rows of use each.
#pragma once

#include "gemm2_bf16.h"
#include "merge_scatter_bf16.h"

namespace lory {
namespace fmg {

using gemm::bf16x8;
using gemm::f32x16;
using gemm::s16x4;
using gemm::u32x2;
using gemm::u32x4;
using ms::Frag;

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int BN = 64;        // output columns of a task
constexpr int BK = 32;        // K step of the token ring (two 16-wide slices)
constexpr int kSegBytes = 2048;  // merged 16 x 64 bf16 tile of one segment

struct Params {
    const uint16_t *A[2];   // token operands [tokens][lda], K contiguous, one per source
    int lda[2];
    const uint16_t *W[2];   // expert stacks, one per source, already offset to the first column / row used
    long expert_stride;     // elements between experts
    int ldw;                // elements between rows of one expert matrix
    const float *w;         // routing weights [S][E]
    int E, T;
    int tokens;             // rows of A and C
    int N, K;               // output columns (multiple of 64); contraction length per source (multiple of 32)
    uint16_t *C;            // [tokens][ldc]
    int ldc;
};

// KG: the merged tiles are formed per K step (32 wide) instead of per slice (16 wide).
template <int WROWS, int SPW, bool KG>
struct Smem {
    static constexpr int a_stage = WROWS * 64;              // one K step of one wave's rows
    static constexpr int a_bytes = 4 * 2 * a_stage;         // four waves, two stages
    static constexpr int seg_bytes = KG ? 2 * kSegBytes : kSegBytes;
    static constexpr int m_bytes = 4 * SPW * seg_bytes;     // one merged tile of all segments of the task
    static constexpr int total = a_bytes + 2 * m_bytes;
};

// W_NC: expert matrices stored [K][N] (N contiguous: forward projections); else [N][K] (K contiguous:
// the transposed uses of the backward).  SPW = WROWS / T segments per wavefront.
// E16 (at most 16 experts and 8 segments per task): one merge MFMA covers both units of the wave,
// experts of unit 0 in K 0..15 against rows 0..7, experts of unit 1 in K 16..31 against rows 8..15
// (the routing-weight operand is block diagonal), which halves the expert loads and the merge MFMAs
// and leaves registers for two slices of expert chunks in flight.
// KG (with E16 and K-contiguous expert matrices, where the merged tiles fit): the merge works on whole
// K steps.  A 16-wide slice of a K-contiguous row is only 32 bytes, and fetching rows in 32-byte
// pieces measured 2.5 times as many L2 requests per byte as the forward's 128-byte rows.
template <int WROWS, int SPW, int NSRC, bool W_NC, bool E16, bool KG>
__global__ __launch_bounds__(kThreads, 1) void fmg_kernel(const Params p)
{
    static_assert(!KG || (E16 && !W_NC), "K-step-wide merged tiles: E16, K-contiguous expert matrices");
    using SM = Smem<WROWS, SPW, KG>;
    constexpr int SEGB = SM::seg_bytes;
    constexpr int MI = WROWS / 32;      // 32-row blocks per wave
    constexpr int NI = BN / 32;
    constexpr int SC = 4 * SPW;         // segments per task
    constexpr int R = 4 * WROWS;        // rows per task
    constexpr int RB_SEG = MI / SPW;    // row blocks per segment
    constexpr int NLD = WROWS / 16;     // direct loads per wave and K step
    static_assert(SC <= 16, "the merge MFMA has 16 rows");
    static_assert(!E16 || SC <= 8, "two units share the 16 rows of one merge MFMA");

    extern __shared__ __attribute__((aligned(16))) char smem[];
    typedef __attribute__((address_space(3))) s16x4 *lds_tr_ptr;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const uint32_t wave_u = __builtin_amdgcn_readfirstlane(wave);
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)smem;
    char *a_ring = smem + wave * 2 * SM::a_stage;
    const uint32_t a_ring_u = lds0 + wave_u * 2 * SM::a_stage;
    char *m_buf = smem + SM::a_bytes;

    const int c16 = lane & 15, kg = lane >> 4;   // merge roles: chunk of the unit, expert group / segment group
    const int ksteps = p.K / BK;
    const int G = ksteps * NSRC;                 // K steps of a task
    const int HS = 2 * G;                        // 16-wide slices of a task

    const int nrc = p.tokens / R, ncb = p.N / BN;
    const int rcg = (nrc + 7) >> 3, cbg = (ncb + 3) >> 2;
    const int nsuper = rcg * cbg;
    const int xcd = blockIdx.x & 7, q0 = blockIdx.x >> 3, wg_per_xcd = gridDim.x >> 3;

    // Tasks are dealt in blocks of 8 row chunks x 4 column blocks per XCD (workgroups are placed
    // round-robin on the 8 XCDs): the 32 workgroups of an XCD then share 8 token tiles and 4 sets
    // of expert tiles per K step in their L2, the split that minimises what the XCD fetches.
    for (int sup = xcd; sup < nsuper; sup += 8) {
        for (int q = q0; q < 32; q += wg_per_xcd) {
            const int rc = (sup % rcg) * 8 + (q & 7);
            const int cb = (sup / rcg) * 4 + (q >> 3);
            if (rc >= nrc || cb >= ncb) continue;   // uniform over the workgroup

            const int row0 = rc * R + wave * WROWS;
            const int seg0 = (rc * R) / p.T;
            const int n0 = cb * BN;

            // ---- routing weights as the A operand of the merge MFMA: row = c16, K = 8 kg .. 8 kg + 7.
            //      Plain: row = segment, K = expert.  E16: rows 0..7 = segments against K 0..15 = experts
            //      (unit 0), rows 8..15 = the same segments against K 16..31 = experts (unit 1).
            Frag whi, wlo;
            {
                float v[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int kk = 8 * kg + i;
                    int seg = c16, e = kk;
                    bool ok = true;
                    if constexpr (E16) {
                        seg = c16 & 7;
                        e = kk & 15;
                        ok = (c16 >> 3) == (kk >> 4);
                    }
                    v[i] = (ok && seg < SC && e < p.E) ? p.w[(size_t)(seg0 + seg) * p.E + e] : 0.f;
                }
                ms::split_hi_lo(v, whi, wlo);
            }

            // ---- per-lane addressing of the token ring: LDS chunk position L = 64 i + lane of the wave's
            //      K-contiguous tile is row 16 i + lane / 4, slot lane & 3 (gemm2's swizzle, which only
            //      depends on the low row bits, i.e. on the lane)
            const int arow = lane >> 2;
            const int aslot = (lane & 3) ^ gemm2::fkc(arow);
            long a_off[NSRC];
#pragma unroll
            for (int s = 0; s < NSRC; ++s) a_off[s] = (long)(row0 + arow) * p.lda[s] + (aslot << 3);
            auto issue_a = [&](int g) {
                const int src = (NSRC == 2) ? (g / ksteps) : 0;
                const int ks = (NSRC == 2) ? (g % ksteps) : g;
                const uint16_t *a = p.A[src] + a_off[src] + ks * BK;
                const long step = (long)16 * p.lda[src];
                const uint32_t dst = a_ring_u + (g & 1) * SM::a_stage;
#pragma unroll
                for (int i = 0; i < NLD; ++i) gemm2::dma16(a + i * step, dst + i * 1024);
            };

            // ---- expert chunks of a slice: this wave merges units 2 wave, 2 wave + 1 (16 chunks each)
            //      W_NC:  unit u = K rows 2u, 2u+1 x 8 chunks of 8 columns
            //      else:  unit u = columns 8u .. 8u+7 x 2 chunks of 8 K values
            //      Plain: lane (c16, kg) loads chunk c16 of both units from experts 8 kg .. 8 kg + 7.
            //      E16:   lane (c16, kg) loads chunk c16 of unit kg >> 1 from experts 8 (kg & 1) .. + 7.
            //      KG:    per K step the wave merges its 16 columns x 32 K values in two groups of 8
            //             columns; lane (c16, kg) loads chunk c16 & 3 (8 K values) of column
            //             4 (kg >> 1) + (c16 >> 2) of the group: 64 contiguous bytes per column.
            const long w_unit = KG ? (long)8 * p.ldw : W_NC ? (long)2 * p.ldw : (long)8 * p.ldw;
            long w_lane;   // element offset of this lane's chunk (unit 2 wave, or its own unit), slice 0, expert 0
            if constexpr (KG)
                w_lane = (long)(n0 + 16 * wave + 4 * (kg >> 1) + (c16 >> 2)) * p.ldw + 8 * (c16 & 3);
            else if constexpr (W_NC)
                w_lane = (long)(4 * wave + (c16 >> 3)) * p.ldw + n0 + 8 * (c16 & 7);
            else
                w_lane = (long)(n0 + 16 * wave + (c16 >> 1)) * p.ldw + 8 * (c16 & 1);
            if constexpr (E16 && !KG) w_lane += (kg >> 1) * w_unit;
            {
                const int e0 = E16 ? 8 * (kg & 1) : 8 * kg;
                w_lane += (long)(e0 < p.E ? e0 : 0) * p.expert_stride;   // lanes without experts re-read expert 0 (weight 0)
            }
            const int e_first = E16 ? 8 * (kg & 1) : 8 * kg;
            constexpr int NEX = E16 ? 2 : 1;   // slices of expert chunks in flight
            constexpr int NUL = E16 ? 1 : 2;   // load groups per slice
            Frag EX[NEX][NUL][8];
            // Slice hs into register set buf; KG: column group buf of K step hs.
            auto load_ex = [&](auto buf, int hs) {
                const int g = KG ? hs : (hs >> 1);
                const int src = (NSRC == 2) ? (g / ksteps) : 0;
                const int ks = (NSRC == 2) ? (g % ksteps) : g;
                const int kbase = ks * BK + (KG ? 0 : (hs & 1) * 16);
                const uint16_t *wp = p.W[src] + w_lane + (W_NC ? (long)kbase * p.ldw : (long)kbase);
                if constexpr (KG) wp += buf * w_unit;
#pragma unroll
                for (int ul = 0; ul < NUL; ++ul)
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        // experts beyond E: any valid address (their routing weight is zero)
                        const long eo = (e_first + i < p.E) ? (long)i * p.expert_stride : 0;
                        EX[buf][ul][i].u = *reinterpret_cast<const uint4 *>(wp + ul * w_unit + eo);
                    }
            };
            // merged slice hs -> m_buf[hs & 1]; layout per segment
            //   W_NC: [16 k][64 n], 32-byte granule g of row k at g ^ 2 ((k >> 1) & 1)  (read with the
            //         transposing LDS load: four rows x 64 bytes per half wave, conflict free)
            //   else: [64 n][16 k], 16-byte half h of row n at h ^ ((n >> 3) & 1)
            // Output rows of the merge MFMA held by this lane: 4 kg + r.  Plain: segment 4 kg + r of the
            // unit being processed.  E16: unit kg >> 1, segment 4 (kg & 1) + r.
            //   KG:   [64 n][32 k], 16-byte chunk c of row n at c ^ ((n >> 2) & 3); register set buf holds
            //         column group buf of K step hs
            auto produce = [&](auto buf, int hs) {
                char *mb = m_buf + (hs & 1) * SM::m_bytes;
#pragma unroll
                for (int ul = 0; ul < NUL; ++ul) {
                    Frag P[8];
                    ms::transpose8x8(EX[buf][ul], P);
                    f32x4 macc[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        macc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
                        macc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(whi.v, P[j].v, macc[j], 0, 0, 0);
                        macc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wlo.v, P[j].v, macc[j], 0, 0, 0);
                    }
                    const int uo = E16 ? (kg >> 1) : ul;          // unit (2 wave + uo) these rows belong to
                    const int sbase = E16 ? 4 * (kg & 1) : 4 * kg;
                    int off;
                    if constexpr (KG) {
                        const int nl = 16 * wave + 8 * buf + 4 * uo + (c16 >> 2);
                        off = nl * 64 + (((c16 & 3) ^ ((nl >> 2) & 3)) << 4);
                    } else if constexpr (W_NC) {
                        const int kl = 4 * wave + 2 * uo + (c16 >> 3);
                        const int g32 = ((c16 & 7) >> 1) ^ (uo << 1);
                        off = kl * 128 + (g32 << 5) + ((c16 & 1) << 4);
                    } else {
                        const int nl = 16 * wave + 8 * uo + (c16 >> 1);
                        off = nl * 32 + (((c16 & 1) ^ uo) << 4);
                    }
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int seg = sbase + r;
                        if (seg < SC) {
                            uint4 o;
                            o.x = ms::pack_bf16(macc[0][r], macc[1][r]);
                            o.y = ms::pack_bf16(macc[2][r], macc[3][r]);
                            o.z = ms::pack_bf16(macc[4][r], macc[5][r]);
                            o.w = ms::pack_bf16(macc[6][r], macc[7][r]);
                            *reinterpret_cast<uint4 *>(mb + seg * SEGB + off) = o;
                        }
                    }
                }
            };
            // B operand of the token MFMA: columns jn * 32 .. + 31 of segment sl's merged slice
            auto frag_b = [&](const char *mb, int sl, int jn, int h) -> bf16x8 {
                if constexpr (KG) {
                    const int n = jn * 32 + (lane & 31);
                    const int c = (2 * h + (lane >> 5)) ^ ((n >> 2) & 3);
                    return *reinterpret_cast<const bf16x8 *>(mb + sl * SEGB + n * 64 + (c << 4));
                } else if constexpr (W_NC) {
                    const int g16 = lane >> 4, r = lane & 15;
                    const int coloff = (jn * 32 + 16 * (g16 & 1) + 4 * (r & 3)) * 2;
                    const int krow = 8 * (g16 >> 1) + (r >> 2);
                    const int g32 = (coloff >> 5) ^ (((krow >> 1) & 1) << 1);
                    const char *q = mb + sl * SEGB + krow * 128 + (g32 << 5) + (coloff & 31);
                    union {
                        s16x4 h[2];
                        bf16x8 v;
                    } u;
                    u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_tr_ptr)(q));
                    u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_tr_ptr)(q + 4 * 128));
                    return u.v;
                } else {
                    const int n = jn * 32 + (lane & 31);
                    const int half = (lane >> 5) ^ ((n >> 3) & 1);
                    return *reinterpret_cast<const bf16x8 *>(mb + sl * SEGB + n * 32 + (half << 4));
                }
            };

            f32x16 acc[MI][NI];
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

            // The token MFMAs of slice hs: this wave's rows against the merged tiles of their segments.
            auto multiply = [&](int hs) {
                const int g = hs >> 1, h = hs & 1;
                const char *as = a_ring + (g & 1) * SM::a_stage;
                const char *mb = m_buf + ((KG ? g : hs) & 1) * SM::m_bytes;
#pragma unroll
                for (int sg = 0; sg < SPW; ++sg) {
                    bf16x8 bfr[NI];
#pragma unroll
                    for (int j = 0; j < NI; ++j) bfr[j] = frag_b(mb, wave * SPW + sg, j, h);
#pragma unroll
                    for (int ib = 0; ib < RB_SEG; ++ib) {
                        const int i = sg * RB_SEG + ib;
                        const bf16x8 af = gemm2::frag_kc(as, i * 32, h, lane);
#pragma unroll
                        for (int j = 0; j < NI; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af, acc[i][j], 0, 0, 0);
                    }
                }
            };
            using B0 = std::integral_constant<int, 0>;
            using B1 = std::integral_constant<int, NEX - 1>;

            // ---- schedule.  Slice hs is multiplied while slice hs + 1 is merged (into the other merged
            // buffer) and the expert chunks of slice hs + 1 + NEX are fetched into the registers the
            // merge has just freed.  Token tiles are fetched two K steps ahead, right BEFORE a group of
            // expert loads whose data is consumed before the tile is read: loads retire in order, so
            // the wait the compiler puts in front of that consumption also covers the tile (the direct
            // loads themselves are invisible to its bookkeeping, which makes its waits stricter than
            // needed, never weaker).  (Issuing the tile after the group instead measured slower: the
            // compiler's wait for the PREVIOUS group then also has to retire half of the tile.)
            issue_a(0);
            if (G > 1) issue_a(1);
            if constexpr (KG) {
                // One barrier per K step: both slices of K step g are multiplied from merged tile g
                // while tile g + 1 is merged from the two column groups fetched during K step g - 1.
                load_ex(B0(), 0);
                load_ex(B1(), 0);
                gemm2::wait_vmcnt<0>();
                produce(B0(), 0);
                produce(B1(), 0);
                if (G > 1) {
                    load_ex(B0(), 1);
                    load_ex(B1(), 1);
                }
            } else {
                load_ex(B0(), 0);
                if constexpr (E16) {
                    if (HS > 1) load_ex(B1(), 1);
                }
                gemm2::wait_vmcnt<0>();
                produce(B0(), 0);
                if constexpr (E16) {
                    if (HS > 2) load_ex(B0(), 2);
                } else {
                    if (HS > 1) load_ex(B0(), 1);
                }
            }

            for (int g = 0; KG && g < G; ++g) {
                gemm2::ring_barrier();   // merged tile g complete for every wave; tile g - 1 no longer read
                multiply(2 * g);
                multiply(2 * g + 1);
                if (g + 1 < G) {
                    produce(B0(), g + 1);
                    produce(B1(), g + 1);
                }
                if (g + 2 < G) {
                    __builtin_amdgcn_s_waitcnt(0xC07F);   // this wave's reads of ring slot g & 1 have returned
                    issue_a(g + 2);
                    load_ex(B0(), g + 2);
                    load_ex(B1(), g + 2);
                }
            }

            for (int g = 0; !KG && g < G; ++g) {
                const int hs = 2 * g;
                // ---- even slice
                gemm2::ring_barrier();   // merged slice hs complete for every wave; slice hs - 1 no longer read
                multiply(hs);
                produce(B1(), hs + 1);
                if (hs + 1 + NEX < HS) load_ex(B1(), hs + 1 + NEX);
                // ---- odd slice
                gemm2::ring_barrier();
                multiply(hs + 1);
                if (hs + 2 < HS) produce(B0(), hs + 2);
                if (g + 2 < G) {
                    __builtin_amdgcn_s_waitcnt(0xC07F);   // this wave's reads of ring slot g & 1 have returned
                    issue_a(g + 2);
                }
                if (hs + 2 + NEX < HS) load_ex(B0(), hs + 2 + NEX);
            }

            // ---- epilogue, wave-local: 32-row blocks leave through the wave's own ring memory (all of
            //      its direct loads have landed) as 16-byte stores, 128 bytes contiguous per row.
            //      Accumulator element r of a block: row lane & 31, column 8 (r >> 2) + 4 (lane >> 5) + (r & 3).
            {
                char *stg = a_ring;
                const int r31 = lane & 31, h2 = lane >> 5;
#pragma unroll
                for (int i = 0; i < MI; ++i) {
#pragma unroll
                    for (int j = 0; j < NI; ++j)
#pragma unroll
                        for (int rq = 0; rq < 4; ++rq) {
                            const int nl = j * 32 + 8 * rq + 4 * h2;
                            u32x2 pk;
                            pk.x = gemm::cvt_pk_bf16(acc[i][j][rq * 4 + 0], acc[i][j][rq * 4 + 1]);
                            pk.y = gemm::cvt_pk_bf16(acc[i][j][rq * 4 + 2], acc[i][j][rq * 4 + 3]);
                            const int c = nl >> 3;
                            *reinterpret_cast<u32x2 *>(stg + r31 * 128 + ((c ^ (r31 & 7)) << 4) + h2 * 8) = pk;
                        }
                    __builtin_amdgcn_wave_barrier();
#pragma unroll
                    for (int it = 0; it < 4; ++it) {
                        const int idx = it * 64 + lane;
                        const int row = idx >> 3, c = idx & 7;
                        const u32x4 val = *reinterpret_cast<const u32x4 *>(stg + row * 128 + ((c ^ (row & 7)) << 4));
                        __builtin_nontemporal_store(
                            val, reinterpret_cast<u32x4 *>(p.C + (size_t)(row0 + i * 32 + row) * p.ldc + n0 + c * 8));
                    }
                    __builtin_amdgcn_wave_barrier();
                }
            }
            // the next task's prologue refills ring slot 0 and merged buffer 0: every wave is past the
            // last barrier, after which only buffer 1 and the waves' own ring memory were read
            __builtin_amdgcn_s_waitcnt(0xC07F);
        }
    }
    gemm2::wait_vmcnt<0>();
}

// ---------------------------------------------------------------------------------------------
// Eight-wavefront variant for at most 16 experts: 512 token rows x 64 columns per task, 64 rows and
// 64 accumulator registers per wave, so that two waves share a SIMD and one wave's loads, LDS traffic
// and transposes overlap the other's MFMAs (the four-wave kernel above is alone on its SIMD).
// The merge works on whole K steps (32 wide): per K step every wave merges two 16-chunk units
// (one load group of 8 x 16 bytes per lane, one 16x16x32 MFMA pass with the block-diagonal
// routing-weight operand) for all R / T <= 8 segments of the task; one barrier per K step, two
// multiplied slices between barriers.  Merged tile of a segment: 4 KB,
//   W_NC: [32 k][64 n], 32-byte granule g of row k at g ^ 2 ((k >> 1) & 1)
//   else: [64 n][32 k], 16-byte chunk c of row n at c ^ ((n >> 2) & 3).
template <int TSEG>
struct Smem8 {
    static constexpr int a_stage = 64 * 64;                  // one K step of one wave's 64 rows
    static constexpr int a_bytes = 8 * 2 * a_stage;          // eight waves, two stages
    static constexpr int seg_bytes = 4096;
    static constexpr int m_bytes = (512 / TSEG) * seg_bytes; // one merged K step of all segments of the task
    static constexpr int total = a_bytes + 2 * m_bytes;
};

template <int TSEG, int NSRC, bool W_NC>
__global__ __launch_bounds__(512, 1) void fmg8_kernel(const Params p)
{
    using SM = Smem8<TSEG>;
    constexpr int WROWS = 64, R = 512, MI = 2, NI = 2, NLD = 4;
    constexpr int SC = R / TSEG;
    constexpr int SEGB = SM::seg_bytes;
    static_assert(SC >= 1 && SC <= 8, "two units share the 16 rows of one merge MFMA");

    extern __shared__ __attribute__((aligned(16))) char smem[];
    typedef __attribute__((address_space(3))) s16x4 *lds_tr_ptr;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const uint32_t wave_u = __builtin_amdgcn_readfirstlane(wave);
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)smem;
    char *a_ring = smem + wave * 2 * SM::a_stage;
    const uint32_t a_ring_u = lds0 + wave_u * 2 * SM::a_stage;
    char *m_buf = smem + SM::a_bytes;

    const int c16 = lane & 15, kg = lane >> 4;
    const int ksteps = p.K / BK;
    const int G = ksteps * NSRC;

    const int nrc = p.tokens / R, ncb = p.N / BN;
    const int rcg = (nrc + 7) >> 3, cbg = (ncb + 3) >> 2;
    const int nsuper = rcg * cbg;
    const int xcd = blockIdx.x & 7, q0 = blockIdx.x >> 3, wg_per_xcd = gridDim.x >> 3;

    // same dealing of tasks as the four-wave kernel: 8 row chunks x 4 column blocks per XCD at a time
    for (int sup = xcd; sup < nsuper; sup += 8) {
        for (int q = q0; q < 32; q += wg_per_xcd) {
            const int rc = (sup % rcg) * 8 + (q & 7);
            const int cb = (sup / rcg) * 4 + (q >> 3);
            if (rc >= nrc || cb >= ncb) continue;   // uniform over the workgroup

            const int row0 = rc * R + wave * WROWS;
            const int seg0 = (rc * R) / TSEG;
            const int sl = (wave * WROWS) / TSEG;    // segment (within the task) of this wave's rows
            const int n0 = cb * BN;

            // block-diagonal routing-weight operand: rows 0..7 = segments against K 0..15 = experts
            // (first unit), rows 8..15 = the same segments against K 16..31 = experts (second unit)
            Frag whi, wlo;
            {
                float v[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int kk = 8 * kg + i;
                    const int seg = c16 & 7, e = kk & 15;
                    const bool ok = (c16 >> 3) == (kk >> 4);
                    v[i] = (ok && seg < SC && e < p.E) ? p.w[(size_t)(seg0 + seg) * p.E + e] : 0.f;
                }
                ms::split_hi_lo(v, whi, wlo);
            }

            const int arow = lane >> 2;
            const int aslot = (lane & 3) ^ gemm2::fkc(arow);
            long a_off[NSRC];
#pragma unroll
            for (int s = 0; s < NSRC; ++s) a_off[s] = (long)(row0 + arow) * p.lda[s] + (aslot << 3);
            auto issue_a = [&](int g) {
                const int src = (NSRC == 2) ? (g / ksteps) : 0;
                const int ks = (NSRC == 2) ? (g % ksteps) : g;
                const uint16_t *a = p.A[src] + a_off[src] + ks * BK;
                const long step = (long)16 * p.lda[src];
                const uint32_t dst = a_ring_u + (g & 1) * SM::a_stage;
#pragma unroll
                for (int i = 0; i < NLD; ++i) gemm2::dma16(a + i * step, dst + i * 1024);
            };

            // expert chunks of a K step: lane (c16, kg) loads its chunk of unit kg >> 1 from experts
            // 8 (kg & 1) .. + 7.   W_NC: units = K rows 4 wave + 2 u + {0, 1}, chunk = 8 columns.
            // else: units = columns 8 wave + 4 u + {0..3}, chunk = 8 K values (64 bytes per column).
            // (byte offsets from the K step's first element, 32 bits: the stack is smaller than 2 GiB)
            uint32_t w_lane;
            if constexpr (W_NC)
                w_lane = (uint32_t)(4 * wave + 2 * (kg >> 1) + (c16 >> 3)) * (uint32_t)p.ldw + n0 + 8 * (c16 & 7);
            else
                w_lane = (uint32_t)(n0 + 8 * wave + 4 * (kg >> 1) + (c16 >> 2)) * (uint32_t)p.ldw + 8 * (c16 & 3);
            const int e_first = 8 * (kg & 1);
            const uint32_t stride_b = (uint32_t)p.expert_stride * 2u;
            w_lane = w_lane * 2u + (uint32_t)(e_first < p.E ? e_first : 0) * stride_b;
            Frag EX[8];
            auto load_ex = [&](int g) {
                const int src = (NSRC == 2) ? (g / ksteps) : 0;
                const int ks = (NSRC == 2) ? (g % ksteps) : g;
                const char *wk = reinterpret_cast<const char *>(p.W[src]) +
                                 (W_NC ? (size_t)ks * BK * p.ldw : (size_t)ks * BK) * 2;   // wave-uniform
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const uint32_t off = w_lane + ((e_first + i < p.E) ? (uint32_t)i * stride_b : 0u);   // beyond E: weight 0
                    EX[i].u = *reinterpret_cast<const uint4 *>(wk + off);
                }
            };
            auto produce = [&](int g) {
                char *mb = m_buf + (g & 1) * SM::m_bytes;
                Frag P[8];
                ms::transpose8x8(EX, P);
                const int uo = kg >> 1, sbase = 4 * (kg & 1);   // rows 4 kg + r: unit, segment
                int off;
                if constexpr (W_NC) {
                    const int kl = 4 * wave + 2 * uo + (c16 >> 3);
                    const int g32 = ((c16 & 7) >> 1) ^ (uo << 1);
                    off = kl * 128 + (g32 << 5) + ((c16 & 1) << 4);
                } else {
                    const int nl = 8 * wave + 4 * uo + (c16 >> 2);
                    off = nl * 64 + (((c16 & 3) ^ ((nl >> 2) & 3)) << 4);
                }
                // two halves of the 8 elements of a chunk, to keep fewer merge accumulators alive
#pragma unroll
                for (int hf = 0; hf < 2; ++hf) {
                    f32x4 macc[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        macc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
                        macc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(whi.v, P[4 * hf + j].v, macc[j], 0, 0, 0);
                        macc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wlo.v, P[4 * hf + j].v, macc[j], 0, 0, 0);
                    }
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int seg = sbase + r;
                        if (seg < SC) {
                            uint2 o;
                            o.x = ms::pack_bf16(macc[0][r], macc[1][r]);
                            o.y = ms::pack_bf16(macc[2][r], macc[3][r]);
                            *reinterpret_cast<uint2 *>(mb + seg * SEGB + off + 8 * hf) = o;
                        }
                    }
                }
            };
            auto frag_b = [&](const char *mb, int jn, int h) -> bf16x8 {
                if constexpr (W_NC) {
                    const int g16 = lane >> 4, r = lane & 15;
                    const int coloff = (jn * 32 + 16 * (g16 & 1) + 4 * (r & 3)) * 2;
                    const int krow = 16 * h + 8 * (g16 >> 1) + (r >> 2);
                    const int g32 = (coloff >> 5) ^ (((krow >> 1) & 1) << 1);
                    const char *q = mb + sl * SEGB + krow * 128 + (g32 << 5) + (coloff & 31);
                    union {
                        s16x4 hh[2];
                        bf16x8 v;
                    } u;
                    u.hh[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_tr_ptr)(q));
                    u.hh[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_tr_ptr)(q + 4 * 128));
                    return u.v;
                } else {
                    const int n = jn * 32 + (lane & 31);
                    const int c = (2 * h + (lane >> 5)) ^ ((n >> 2) & 3);
                    return *reinterpret_cast<const bf16x8 *>(mb + sl * SEGB + n * 64 + (c << 4));
                }
            };

            f32x16 acc[MI][NI];
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

            auto multiply = [&](int g, int h) {
                const char *as = a_ring + (g & 1) * SM::a_stage;
                const char *mb = m_buf + (g & 1) * SM::m_bytes;
                bf16x8 bfr[NI];
#pragma unroll
                for (int j = 0; j < NI; ++j) bfr[j] = frag_b(mb, j, h);
#pragma unroll
                for (int i = 0; i < MI; ++i) {
                    const bf16x8 af = gemm2::frag_kc(as, i * 32, h, lane);
#pragma unroll
                    for (int j = 0; j < NI; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af, acc[i][j], 0, 0, 0);
                }
            };

            // Token tiles two K steps ahead, issued right before the expert loads of the same K step,
            // whose data is consumed (by produce) before the tile is read: the compiler's wait in
            // front of that consumption covers the tile (loads retire in order).  (Expert chunks two
            // K steps ahead and a third ring stage measured the same: the kernel is bound by the bytes
            // entering the CU, not by their latency.)
            issue_a(0);
            issue_a(1);
            load_ex(0);
            gemm2::wait_vmcnt<0>();
            produce(0);
            load_ex(1);
            for (int g = 0; g < G; ++g) {   // G is even and at least 2
                gemm2::ring_barrier();   // merged tile g complete for every wave; tile g - 1 no longer read
                multiply(g, 0);
                multiply(g, 1);
                if (g + 1 < G) produce(g + 1);
                if (g + 2 < G) {
                    __builtin_amdgcn_s_waitcnt(0xC07F);   // this wave's reads of ring slot g & 1 have returned
                    issue_a(g + 2);
                    load_ex(g + 2);
                }
            }

            // epilogue through the wave's own ring memory, as in the four-wave kernel
            {
                char *stg = a_ring;
                const int r31 = lane & 31, h2 = lane >> 5;
#pragma unroll
                for (int i = 0; i < MI; ++i) {
#pragma unroll
                    for (int j = 0; j < NI; ++j)
#pragma unroll
                        for (int rq = 0; rq < 4; ++rq) {
                            const int nl = j * 32 + 8 * rq + 4 * h2;
                            u32x2 pk;
                            pk.x = gemm::cvt_pk_bf16(acc[i][j][rq * 4 + 0], acc[i][j][rq * 4 + 1]);
                            pk.y = gemm::cvt_pk_bf16(acc[i][j][rq * 4 + 2], acc[i][j][rq * 4 + 3]);
                            const int c = nl >> 3;
                            *reinterpret_cast<u32x2 *>(stg + r31 * 128 + ((c ^ (r31 & 7)) << 4) + h2 * 8) = pk;
                        }
                    __builtin_amdgcn_wave_barrier();
#pragma unroll
                    for (int it = 0; it < 4; ++it) {
                        const int idx = it * 64 + lane;
                        const int row = idx >> 3, c = idx & 7;
                        const u32x4 val = *reinterpret_cast<const u32x4 *>(stg + row * 128 + ((c ^ (row & 7)) << 4));
                        __builtin_nontemporal_store(
                            val, reinterpret_cast<u32x4 *>(p.C + (size_t)(row0 + i * 32 + row) * p.ldc + n0 + c * 8));
                    }
                    __builtin_amdgcn_wave_barrier();
                }
            }
            __builtin_amdgcn_s_waitcnt(0xC07F);
        }
    }
    gemm2::wait_vmcnt<0>();
}

// whole tasks and an even number of K steps, as for the four-wave kernel
template <int TSEG>
inline bool fits8(const Params &p)
{
    return p.T == TSEG && p.tokens % 512 == 0 && p.N % BN == 0 && p.K % (2 * BK) == 0 && p.E <= 16 && p.E >= 1 &&
           (size_t)p.E * (size_t)p.expert_stride * 2 < ((size_t)1 << 31);
}

template <int TSEG, int NSRC, bool W_NC>
inline hipError_t launch8(const Params &p, hipStream_t st)
{
    using SM = Smem8<TSEG>;
    static_assert(SM::total <= 160 * 1024, "LDS of one CU");
    auto kern = fmg8_kernel<TSEG, NSRC, W_NC>;
    static bool configured = false;  // per instantiation
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, SM::total);
        if (e != hipSuccess) return e;
        configured = true;
    }
    const long tasks = (long)(p.tokens / 512) * (p.N / BN);
    long blocks = (tasks + 7) / 8 * 8;
    if (blocks > gemm2::persistent_grid()) blocks = gemm2::persistent_grid();
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(512), SM::total, st, p);
    return hipGetLastError();
}

// Shapes the kernel takes: whole tasks only, and an even number of K steps (a task's last merged tile
// then sits in buffer 1, which the next task's prologue leaves alone).
template <int WROWS, int SPW>
inline bool fits(const Params &p)
{
    return p.T * SPW == WROWS && p.tokens % (4 * WROWS) == 0 && p.N % BN == 0 && p.K % (2 * BK) == 0 && p.E <= 32 &&
           p.E >= 1;
}

template <int WROWS, int SPW, int NSRC, bool W_NC, bool E16, bool KG>
inline hipError_t launch_t(const Params &p, hipStream_t st)
{
    using SM = Smem<WROWS, SPW, KG>;
    static_assert(SM::total <= 160 * 1024, "LDS of one CU");
    auto kern = fmg_kernel<WROWS, SPW, NSRC, W_NC, E16, KG>;
    static bool configured = false;  // per instantiation
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, SM::total);
        if (e != hipSuccess) return e;
        configured = true;
    }
    const long tasks = (long)(p.tokens / (4 * WROWS)) * (p.N / BN);
    long blocks = (tasks + 7) / 8 * 8;
    if (blocks > gemm2::persistent_grid()) blocks = gemm2::persistent_grid();
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(kThreads), SM::total, st, p);
    return hipGetLastError();
}

template <int WROWS, int SPW, int NSRC, bool W_NC>
inline hipError_t launch(const Params &p, hipStream_t st)
{
    if constexpr (4 * SPW <= 8) {
        if (p.E <= 16) {
            if constexpr (!W_NC && Smem<WROWS, SPW, true>::total <= 160 * 1024)
                return launch_t<WROWS, SPW, NSRC, W_NC, true, true>(p, st);
            else
                return launch_t<WROWS, SPW, NSRC, W_NC, true, false>(p, st);
        }
    }
    return launch_t<WROWS, SPW, NSRC, W_NC, false, false>(p, st);
}

}  // namespace fmg
}  // namespace lory
