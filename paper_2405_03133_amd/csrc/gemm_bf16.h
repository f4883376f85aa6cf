// Batched bf16 MFMA GEMM core for gfx950 (one batch item = one segment of the
// Lory layer).  Every dense contraction of the merged FFN and of its backward
// (paper Section 3.1: o_x = FFN(h_x; theta_bar) for all tokens of a segment;
// Appendix B counts them as 6*L*d*d' FLOPs) is an instance of
//
//     C_b[M,N] = sum over sources q of  A_{q,b}[M,K] * B_{q,b}[K,N]
//
// with fp32 accumulation on v_mfma_f32_32x32x16_bf16.
//
// Operand layouts, chosen per instance by template flags:
//   A: "KC" = stored [M][K] (K contiguous)   or "MC" = stored [K][M]
//   B: "KC" = stored [N][K] (K contiguous)   or "NC" = stored [K][N]
// KC tiles sit in LDS as rows of 64 bf16 with an XOR swizzle of their 16-byte
// chunks and are read with ds_read_b128.  MC/NC tiles sit in LDS as they are
// in memory (rows of the non-contracted index, padded pitch) and are read with
// ds_read_b64_tr_b16, which hands each lane four consecutive K values of its
// own column, i.e. the transposition happens inside the LDS read.
//
// A workgroup is 256 threads = 4 wavefronts computing a BM x BN tile (times
// NSET operand sets that share A, e.g. the gate and up projections).  K is
// walked in steps of 64 with two LDS stages: global loads of step i+1 are
// issued into registers before the MFMAs of step i and stored to the other
// stage afterwards, one barrier per step.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

namespace lory {
namespace gemm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kThreads = 256;
constexpr int BK = 64;

struct Params {
    const uint16_t *A[2];  // per source
    long a_batch[2];       // elements between consecutive batch items
    int lda[2];            // elements between consecutive rows of the stored matrix
    const uint16_t *B[2];  // per operand set (NSET == 2) or per source (NSRC == 2)
    long b_batch[2];
    int ldb[2];
    int M, N, K;           // per batch item; K per source
    int batches;
};

__host__ __device__ constexpr int tr_pitch(int width) { return width * 2 + 64; }

template <int BM, int BN, int NSET, bool A_MC, bool B_NC>
struct Smem {
    static constexpr int a_bytes = A_MC ? BK * tr_pitch(BM) : BM * 128;
    static constexpr int b_bytes = B_NC ? BK * tr_pitch(BN) : BN * 128;
    static constexpr int stage = a_bytes + NSET * b_bytes;
    static constexpr int out_pitch = BN * 2 + 16;     // bytes per row of the epilogue staging tile
    static constexpr int out_bytes = BM * out_pitch;
    static constexpr int total = (2 * stage > out_bytes) ? 2 * stage : out_bytes;
};

// Swizzle of the 16-byte chunk index inside a 128-byte KC row.
__device__ __forceinline__ int swz(int row) { return (row & 7) ^ ((row >> 3) & 1); }

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b)
{
    return __uint_as_float(((uint32_t)b) << 16);
}

// Round to nearest even; inputs here are finite.
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Two floats -> two bf16 (round to nearest even) packed into 32 bits, low half first: a single
// v_cvt_pk_bf16_f32 on gfx950.
__device__ __forceinline__ uint32_t cvt_pk_bf16(float lo, float hi)
{
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const f32x2 v = {lo, hi};
    union {
        bf16x2 b;
        uint32_t u;
    } r;
    r.b = __builtin_convertvector(v, bf16x2);
    return r.u;
}

// ---- global -> register -> LDS staging of one K step --------------------------
//
// KC tile (ROWS rows of 64 bf16): thread t moves chunk (t & 7) of rows (t >> 3) + 32 i.
// TR tile (64 K rows of WIDTH bf16): thread t moves chunks t + 256 i of the row-major tile.

template <int ROWS>
__device__ __forceinline__ void load_kc(u32x4 (&v)[ROWS / 32], const uint16_t *base, int ld, int row0,
                                        int k0, int tid)
{
    const int c = tid & 7;
#pragma unroll
    for (int i = 0; i < ROWS / 32; ++i) {
        const int row = (tid >> 3) + 32 * i;
        v[i] = *reinterpret_cast<const u32x4 *>(base + (size_t)(row0 + row) * ld + k0 + c * 8);
    }
}

template <int ROWS>
__device__ __forceinline__ void store_kc(const u32x4 (&v)[ROWS / 32], char *lds, int tid)
{
    const int c = tid & 7;
#pragma unroll
    for (int i = 0; i < ROWS / 32; ++i) {
        const int row = (tid >> 3) + 32 * i;
        *reinterpret_cast<u32x4 *>(lds + row * 128 + ((c ^ swz(row)) << 4)) = v[i];
    }
}

template <int WIDTH>
__device__ __forceinline__ void load_tr(u32x4 (&v)[WIDTH / 32], const uint16_t *base, int ld, int col0,
                                        int k0, int tid)
{
    constexpr int cpr = WIDTH / 8;  // 16-byte chunks per row
#pragma unroll
    for (int i = 0; i < WIDTH / 32; ++i) {
        const int idx = tid + kThreads * i;
        const int row = idx / cpr, c = idx % cpr;
        v[i] = *reinterpret_cast<const u32x4 *>(base + (size_t)(k0 + row) * ld + col0 + c * 8);
    }
}

template <int WIDTH>
__device__ __forceinline__ void store_tr(const u32x4 (&v)[WIDTH / 32], char *lds, int tid)
{
    constexpr int cpr = WIDTH / 8;
#pragma unroll
    for (int i = 0; i < WIDTH / 32; ++i) {
        const int idx = tid + kThreads * i;
        const int row = idx / cpr, c = idx % cpr;
        *reinterpret_cast<u32x4 *>(lds + row * tr_pitch(WIDTH) + (c << 4)) = v[i];
    }
}

// ---- LDS -> MFMA operand fragments ------------------------------------------

// 32 rows x 16 K of a KC tile: lane holds row (lane & 31), K = kk*16 + (lane>>5)*8 .. +7.
__device__ __forceinline__ bf16x8 frag_kc(const char *lds, int row0, int kk, int lane)
{
    const int row = row0 + (lane & 31);
    const int c = kk * 2 + (lane >> 5);
    return *reinterpret_cast<const bf16x8 *>(lds + row * 128 + ((c ^ swz(row)) << 4));
}

// 32 columns x 16 K of an MC/NC tile through the transposing LDS read.  Within
// a group of 16 lanes, lane r supplies the address of row (r>>2), columns
// 4*(r&3)..+3 of a 4x16 block and receives the 4 rows of column r.  Two reads
// (rows +0..3 and +4..7) give the same K set per lane as frag_kc.
template <int PITCH>
__device__ __forceinline__ bf16x8 frag_tr(const char *lds, int col0, int kk, int lane)
{
    typedef __attribute__((address_space(3))) s16x4 *lds_ptr;
    const int g = lane >> 4, r = lane & 15;
    const int col = col0 + 16 * (g & 1) + 4 * (r & 3);
    const int krow = kk * 16 + 8 * (g >> 1) + (r >> 2);
    const char *p = lds + krow * PITCH + col * 2;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + 4 * PITCH));
    union {
        s16x4 h[2];
        bf16x8 v;
    } u;
    u.h[0] = lo;
    u.h[1] = hi;
    return u.v;
}

// ---- the kernel ---------------------------------------------------------------
//
// The MFMA is issued with the B fragment as its first operand, so a lane ends
// up with one row m and, per accumulator quad, four consecutive columns n.
//
// Epi describes the epilogue (fused elementwise work and the output planes):
//   Epi::NOUT                  number of output planes (bf16 matrices)
//   Epi::In  / epi.load(b,m,n) optional per-quad inputs (four consecutive n)
//   epi.enabled(o)             whether plane o is written at all
//   epi.pack(o, b, m, n, in, v) the four bf16 outputs of plane o for the quad at (m, n..n+3), v[NSET][4] fp32
//   epi.ptr(o, b, m, n)        global address of element (m, n) of plane o
// Each plane is staged through LDS and leaves the workgroup as 16-byte stores
// that are contiguous along n.
template <int BM, int BN, int WAVES_M, int NSET, int NSRC, bool A_MC, bool B_NC, class Epi>
__global__ __launch_bounds__(kThreads, 1) void gemm_kernel(const Params p, const Epi epi)
{
    static_assert(NSET == 1 || NSRC == 1, "either two operand sets or two sources");
    constexpr int WAVES_N = 4 / WAVES_M;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int MI = WM / 32, NI = WN / 32;
    static_assert(MI >= 1 && NI >= 1, "wave tile must hold at least one 32x32 block");
    using SM = Smem<BM, BN, NSET, A_MC, B_NC>;
    constexpr int A_PITCH = tr_pitch(BM), B_PITCH = tr_pitch(BN);

    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm0 = (wave / WAVES_N) * WM;
    const int wn0 = (wave % WAVES_N) * WN;

    const int tiles_n = p.N / BN;
    const int tiles_m = p.M / BM;
    int bid = blockIdx.x;
    const int nt = bid % tiles_n;
    bid /= tiles_n;
    const int mt = bid % tiles_m;
    const int batch = bid / tiles_m;
    const int m0 = mt * BM, n0 = nt * BN;

    const int ktiles = p.K / BK;
    const int total_tiles = ktiles * NSRC;

    f32x16 acc[NSET][MI][NI];
#pragma unroll
    for (int s = 0; s < NSET; ++s)
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[s][i][j][r] = 0.f;

    u32x4 ra[BM / 32];
    u32x4 rb[NSET][BN / 32];

#define LORY_LOAD_TILE(t_)                                                                     \
    do {                                                                                       \
        const int src_ = (NSRC == 2) ? ((t_) / ktiles) : 0;                                    \
        const int k0_ = ((t_) % ktiles) * BK;                                                  \
        const uint16_t *a_ = p.A[src_] + (size_t)batch * p.a_batch[src_];                      \
        if constexpr (A_MC)                                                                    \
            load_tr<BM>(ra, a_, p.lda[src_], m0, k0_, tid);                                    \
        else                                                                                   \
            load_kc<BM>(ra, a_, p.lda[src_], m0, k0_, tid);                                    \
        _Pragma("unroll") for (int s_ = 0; s_ < NSET; ++s_)                                    \
        {                                                                                      \
            const int bi_ = (NSRC == 2) ? src_ : s_;                                           \
            const uint16_t *b_ = p.B[bi_] + (size_t)batch * p.b_batch[bi_];                    \
            if constexpr (B_NC)                                                                \
                load_tr<BN>(rb[s_], b_, p.ldb[bi_], n0, k0_, tid);                             \
            else                                                                               \
                load_kc<BN>(rb[s_], b_, p.ldb[bi_], n0, k0_, tid);                             \
        }                                                                                      \
    } while (0)

#define LORY_STORE_TILE(stage_)                                                                \
    do {                                                                                       \
        char *base_ = smem + (stage_) * SM::stage;                                             \
        if constexpr (A_MC)                                                                    \
            store_tr<BM>(ra, base_, tid);                                                      \
        else                                                                                   \
            store_kc<BM>(ra, base_, tid);                                                      \
        _Pragma("unroll") for (int s_ = 0; s_ < NSET; ++s_)                                    \
        {                                                                                      \
            if constexpr (B_NC)                                                                \
                store_tr<BN>(rb[s_], base_ + SM::a_bytes + s_ * SM::b_bytes, tid);             \
            else                                                                               \
                store_kc<BN>(rb[s_], base_ + SM::a_bytes + s_ * SM::b_bytes, tid);             \
        }                                                                                      \
    } while (0)

    LORY_LOAD_TILE(0);
    LORY_STORE_TILE(0);
    __syncthreads();

    for (int t = 0; t < total_tiles; ++t) {
        const bool more = (t + 1 < total_tiles);
        if (more) LORY_LOAD_TILE(t + 1);
        const char *base = smem + (t & 1) * SM::stage;
        const char *la = base;
        const char *lb = base + SM::a_bytes;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8 af[MI];
            bf16x8 bf[NSET][NI];
#pragma unroll
            for (int i = 0; i < MI; ++i) {
                if constexpr (A_MC)
                    af[i] = frag_tr<A_PITCH>(la, wm0 + i * 32, kk, lane);
                else
                    af[i] = frag_kc(la, wm0 + i * 32, kk, lane);
            }
#pragma unroll
            for (int s = 0; s < NSET; ++s)
#pragma unroll
                for (int j = 0; j < NI; ++j) {
                    if constexpr (B_NC)
                        bf[s][j] = frag_tr<B_PITCH>(lb + s * SM::b_bytes, wn0 + j * 32, kk, lane);
                    else
                        bf[s][j] = frag_kc(lb + s * SM::b_bytes, wn0 + j * 32, kk, lane);
                }
#pragma unroll
            for (int s = 0; s < NSET; ++s)
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int j = 0; j < NI; ++j)
                        acc[s][i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[s][j], af[i],
                                                                               acc[s][i][j], 0, 0, 0);
        }
        if (more) LORY_STORE_TILE((t + 1) & 1);
        __syncthreads();
    }
#undef LORY_LOAD_TILE
#undef LORY_STORE_TILE

    // Accumulator element r of a 32x32 block now is row m = lane & 31 and column
    // n = 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3).  The loop above ended with a barrier, so
    // the pipeline stages in LDS are free to hold the output tile.
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
        constexpr int cpr = BN / 8;
#pragma unroll 4
        for (int idx = tid; idx < BM * cpr; idx += kThreads) {
            const int row = idx / cpr, c = idx % cpr;
            const u32x4 val = *reinterpret_cast<const u32x4 *>(smem + row * SM::out_pitch + c * 16);
            *reinterpret_cast<u32x4 *>(epi.ptr(o, batch, m0 + row, n0 + c * 8)) = val;
        }
        __syncthreads();
    }
}

template <int BM, int BN, int WAVES_M, int NSET, int NSRC, bool A_MC, bool B_NC, class Epi>
inline hipError_t launch(const Params &p, const Epi &epi, hipStream_t st)
{
    using SM = Smem<BM, BN, NSET, A_MC, B_NC>;
    auto kern = gemm_kernel<BM, BN, WAVES_M, NSET, NSRC, A_MC, B_NC, Epi>;
    static bool configured = false;  // per instantiation
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, SM::total);
        if (e != hipSuccess) return e;
        configured = true;
    }
    const long blocks = (long)p.batches * (p.M / BM) * (p.N / BN);
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(kThreads), SM::total, st, p, epi);
    return hipGetLastError();
}

}  // namespace gemm
}  // namespace lory
