// Dense SwiGLU FFN with per-sequence merged parameters: the generation phase of
// prompt-only routing (paper Section 3.1, "Prompt-only routing during
// inference"; Appendix G.1).  After one routing decision per layer the merged
// FFN of a sequence is an ordinary dense FFN,
//   Y_b = (silu(X_b Wg_bar_b) (.) X_b Wu_bar_b) Wd_bar_b .
// Long token blocks (bf16, a multiple of 64 tokens per sequence) go through the
// batched MFMA GEMMs.  Everything else (decode steps of one or a few tokens,
// fp32, ragged token counts) goes through the "skinny" kernels below, which are
// HBM-bound: every weight is read once per pass of up to 8 tokens.
//
// Skinny pass, per matrix product out[t][n] = sum_k x[t][k] W[k][n], W row-major:
//   grid (column blocks, K splits, sequences); a wavefront covers 64 * VEC
//   consecutive columns with one 16-byte load per lane and row; the 4 wavefronts
//   of a workgroup take interleaved rows of its K slice; x is staged in LDS as
//   fp32; partial sums go to [K split][sequence][matrix][token][n] in the
//   workspace and are added in split order by their consumer (the down pass forms
//   the SwiGLU activation from the gate/up parts while staging its x; a small
//   finishing kernel adds the down parts and stores Y) => bit-reproducible.
#include "lory_internal.h"

#include "elem_io.h"

namespace lory {

namespace {

constexpr int kSkThreads = 256;
constexpr int kMaxTok = 8;        // tokens per skinny pass
constexpr int kMaxSlice = 512;    // rows of W per workgroup (x slice in LDS: 8 * 512 floats)

template <typename T> using Ld = Elem<T>;

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(__hip_bfloat16 v) { return Ld<__hip_bfloat16>::one(&v); }

// TW: storage type of the weights.  MT tokens, NMAT matrices sharing x (2 = gate and up), VEC
// columns per lane (Ld<TW>::vec, or 1 when N is not a multiple of it).
//   x:    NMAT == 2: the layer input [B][x_rows][K] of type TW (token t of sequence b at
//         x + (b * x_rows + t) * K).  NMAT == 1 (down projection): x is the SwiGLU activation,
//         which is formed on the fly from the gate/up partial sums gu [gu_ks][B][2][MT][K]:
//         silu(sum of gate parts) * (sum of up parts), parts added in split order.
//   W0/1: [B][K][N]
//   part: [ksplit][B][NMAT][MT][N] fp32
template <typename TW, int MT, int NMAT, int VEC>
__global__ __launch_bounds__(kSkThreads) void skinny_kernel(const TW *__restrict__ x, long x_rows,
                                                            const float *__restrict__ gu, int gu_ks,
                                                            const TW *__restrict__ W0,
                                                            const TW *__restrict__ W1, float *__restrict__ part,
                                                            int K, int N, int slice)
{
    __shared__ float xs[kMaxTok * kMaxSlice];
    __shared__ float red[3][64 * VEC];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b = blockIdx.z, B = gridDim.z;
    const int k0 = blockIdx.y * slice;
    const int k1 = (k0 + slice < K) ? (k0 + slice) : K;
    const int c = (blockIdx.x * 64 + lane) * VEC;

    for (int i = tid; i < MT * (k1 - k0); i += kSkThreads) {
        const int t = i / (k1 - k0), k = i - t * (k1 - k0);
        if constexpr (NMAT == 2) {
            xs[t * kMaxSlice + k] = to_f32(x[((size_t)b * x_rows + t) * K + k0 + k]);
        } else {
            const float *pg = gu + ((size_t)b * 2 * MT + t) * K + k0 + k;   // split 0, gate
            const size_t pitch = (size_t)B * 2 * MT * K, up = (size_t)MT * K;
            float g = 0.f, u = 0.f;
            int ks = 0;
            for (; ks + 4 <= gu_ks; ks += 4) {  // loads overlap, adds stay in split order
                float vg[4], vu[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    vg[j] = pg[(size_t)(ks + j) * pitch];
                    vu[j] = pg[(size_t)(ks + j) * pitch + up];
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    g += vg[j];
                    u += vu[j];
                }
            }
            for (; ks < gu_ks; ++ks) {
                g += pg[(size_t)ks * pitch];
                u += pg[(size_t)ks * pitch + up];
            }
            xs[t * kMaxSlice + k] = g / (1.0f + expf(-g)) * u;
        }
    }
    __syncthreads();

    float acc[NMAT][MT][VEC];
#pragma unroll
    for (int a = 0; a < NMAT; ++a)
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[a][t][i] = 0.f;

    if (c < N) {
        const TW *Wb[2] = {W0 + (size_t)b * K * N + c, NMAT == 2 ? W1 + (size_t)b * K * N + c : nullptr};
#pragma unroll 4
        for (int k = k0 + wave; k < k1; k += 4) {
            float wv[NMAT][VEC];
#pragma unroll
            for (int a = 0; a < NMAT; ++a) {
                if constexpr (VEC == 1)
                    wv[a][0] = Ld<TW>::one(Wb[a] + (size_t)k * N);
                else
                    Ld<TW>::load(Wb[a] + (size_t)k * N, wv[a]);
            }
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                const float xv = xs[t * kMaxSlice + (k - k0)];
#pragma unroll
                for (int a = 0; a < NMAT; ++a)
#pragma unroll
                    for (int i = 0; i < VEC; ++i) acc[a][t][i] = fmaf(xv, wv[a][i], acc[a][t][i]);
            }
        }
    }

    // the four wavefronts' sums, added in wavefront order by wavefront 0
    float *dst = part + (((size_t)blockIdx.y * B + b) * NMAT) * MT * N;
#pragma unroll
    for (int a = 0; a < NMAT; ++a)
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            if (wave > 0) {
#pragma unroll
                for (int i = 0; i < VEC; ++i) red[wave - 1][lane * VEC + i] = acc[a][t][i];
            }
            __syncthreads();
            if (wave == 0 && c < N) {
#pragma unroll
                for (int i = 0; i < VEC; ++i) {
                    float v = acc[a][t][i];
                    v += red[0][lane * VEC + i];
                    v += red[1][lane * VEC + i];
                    v += red[2][lane * VEC + i];
                    dst[((size_t)a * MT + t) * N + c + i] = v;
                }
            }
            __syncthreads();
        }
}

// Y[b][t0 + t][j] = sum over the K splits, in split order.   part: [ks][B][1][mt][N]
// One wavefront-wide group of 8 lanes per output element would change the order; instead every
// thread keeps its element and fetches eight parts at a time, so the loads overlap and the adds
// stay sequential.
template <typename T>
__global__ void skinny_finish_down_kernel(const float *__restrict__ part, T *__restrict__ Y, int ksplit, int B,
                                          int mt, int N, long y_rows, int t0)
{
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const long total = (long)B * mt * N;
    if (i >= total) return;
    const int n = (int)(i % N);
    const int t = (int)((i / N) % mt);
    const int b = (int)(i / ((long)N * mt));
    const float *src = part + ((size_t)b * mt + t) * N + n;
    const size_t pitch = (size_t)B * mt * N;
    float y = 0.f;
    int ks = 0;
    for (; ks + 8 <= ksplit; ks += 8) {
        float v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = src[(size_t)(ks + j) * pitch];
#pragma unroll
        for (int j = 0; j < 8; ++j) y += v[j];
    }
    for (; ks < ksplit; ++ks) y += src[(size_t)ks * pitch];
    Ld<T>::store(Y + ((size_t)b * y_rows + t0 + t) * N + n, y);
}

// K splits: enough workgroups to fill the chip, slices of at most kMaxSlice rows.
int choose_ksplit(int K, int N, int B, int vec)
{
    const int colblocks = (N + 64 * vec - 1) / (64 * vec);
    int ks = (1024 + colblocks * B - 1) / (colblocks * B);
    const int min_ks = (K + kMaxSlice - 1) / kMaxSlice;
    if (ks < min_ks) ks = min_ks;
    const int max_ks = (K + 15) / 16;  // at least 16 rows per slice
    if (ks > max_ks) ks = max_ks;
    if (ks < 1) ks = 1;
    return ks;
}

struct SkinnyPlan {
    int vec1, vec2;     // columns per lane in the two phases
    int ks1, ks2;       // K splits
    size_t part1;       // floats of the gate/up partial sums
    size_t part2;       // floats of the down-projection partial sums
};

template <typename T>
SkinnyPlan skinny_plan(const Dims &m)
{
    SkinnyPlan p;
    p.vec1 = (m.dff % Ld<T>::vec == 0) ? Ld<T>::vec : 1;
    p.vec2 = (m.d % Ld<T>::vec == 0) ? Ld<T>::vec : 1;
    p.ks1 = choose_ksplit(m.d, m.dff, m.B, p.vec1);
    p.ks2 = choose_ksplit(m.dff, m.d, m.B, p.vec2);
    const int mt = m.L < kMaxTok ? m.L : kMaxTok;   // tokens of the largest pass
    p.part1 = (size_t)p.ks1 * m.B * 2 * mt * m.dff;
    p.part2 = (size_t)p.ks2 * m.B * mt * m.d;
    return p;
}

template <typename TW, int NMAT, int VEC>
void launch_skinny(hipStream_t st, int mt, dim3 grid, const TW *x, long x_rows, const float *gu, int gu_ks,
                   const TW *W0, const TW *W1, float *part, int K, int N, int slice)
{
#define LORY_SK(M)                                                                                          \
    hipLaunchKernelGGL((skinny_kernel<TW, M, NMAT, VEC>), grid, dim3(kSkThreads), 0, st, x, x_rows, gu,    \
                       gu_ks, W0, W1, part, K, N, slice)
    switch (mt) {
    case 1: LORY_SK(1); break;
    case 2: LORY_SK(2); break;
    case 3: LORY_SK(3); break;
    case 4: LORY_SK(4); break;
    case 5: LORY_SK(5); break;
    case 6: LORY_SK(6); break;
    case 7: LORY_SK(7); break;
    default: LORY_SK(8); break;
    }
#undef LORY_SK
}

template <typename T>
int skinny_ffn(const Dims &m, const T *X, const T *Wbar, T *Y, void *ws, hipStream_t st)
{
    const SkinnyPlan pl = skinny_plan<T>(m);
    float *part1 = (float *)ws;
    float *part2 = part1 + pl.part1;
    const T *Wg = Wbar, *Wu = Wbar + (size_t)m.B * m.D, *Wd = Wbar + (size_t)2 * m.B * m.D;
    const int slice1 = (m.d + pl.ks1 - 1) / pl.ks1, slice2 = (m.dff + pl.ks2 - 1) / pl.ks2;
    const int ks1 = (m.d + slice1 - 1) / slice1, ks2 = (m.dff + slice2 - 1) / slice2;
    const double esz = sizeof(T);
    for (int t0 = 0; t0 < m.L; t0 += kMaxTok) {
        const int mt = (m.L - t0 < kMaxTok) ? (m.L - t0) : kMaxTok;
        prof::Range r(st, prof::kDenseSkinny, 6.0 * m.B * mt * (double)m.D,
                      esz * (3.0 * m.B * m.D + 2.0 * m.B * mt * m.d));
        // phase 1: gate and up partial sums
        {
            const dim3 grid((m.dff + 64 * pl.vec1 - 1) / (64 * pl.vec1), ks1, m.B);
            const T *x = X + (size_t)t0 * m.d;
            if (pl.vec1 == 1)
                launch_skinny<T, 2, 1>(st, mt, grid, x, m.L, nullptr, 0, Wg, Wu, part1, m.d, m.dff, slice1);
            else
                launch_skinny<T, 2, Ld<T>::vec>(st, mt, grid, x, m.L, nullptr, 0, Wg, Wu, part1, m.d, m.dff,
                                                slice1);
        }
        // phase 2: SwiGLU of the summed parts while staging, down projection, then the final sum
        {
            const dim3 grid((m.d + 64 * pl.vec2 - 1) / (64 * pl.vec2), ks2, m.B);
            if (pl.vec2 == 1)
                launch_skinny<T, 1, 1>(st, mt, grid, (const T *)nullptr, 0, part1, ks1, Wd, (const T *)nullptr,
                                       part2, m.dff, m.d, slice2);
            else
                launch_skinny<T, 1, Ld<T>::vec>(st, mt, grid, (const T *)nullptr, 0, part1, ks1, Wd,
                                                (const T *)nullptr, part2, m.dff, m.d, slice2);
            const long n = (long)m.B * mt * m.d;
            hipLaunchKernelGGL((skinny_finish_down_kernel<T>), dim3((unsigned)((n + 255) / 256)), dim3(256), 0,
                               st, part2, Y, ks2, m.B, mt, m.d, (long)m.L, t0);
        }
        if (hipGetLastError() != hipSuccess) return LORY_ERR_DEVICE;
    }
    return LORY_OK;
}

bool gemm_path(const Dims &m) { return m.dtype == LORY_BF16 && m.L % 64 == 0; }

// Scratch of lory_dense_ffn_fwd_static: the partial sums (or the activation block) that
// lory_dense_ffn_fwd keeps in the caller's workspace, held by the library instead.  Every GPU
// the library runs on holds its own copy of the array at its own address until the process
// ends; in host code the array's name is only a handle for hipGetSymbolAddress, the address
// looked up per device is what launches receive.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
void *g_scratch_addr[kMaxDevices];  // device address of `scratch` per device ordinal, looked up once

int static_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LORY_ERR_DEVICE;
    if (!g_scratch_addr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return LORY_ERR_DEVICE;
        g_scratch_addr[dev] = ptr;
    }
    *out = g_scratch_addr[dev];
    return LORY_OK;
}

}  // namespace

size_t dense_static_scratch_limit() { return kStaticScratchBytes; }

int dense_ffn_fwd_static(const Dims &m, const void *X, const void *Wbar, void *Y, hipStream_t st)
{
    if (dense_workspace_bytes(m) > kStaticScratchBytes) return LORY_ERR_WORKSPACE;
    void *ws = nullptr;
    const int rc = static_scratch(&ws);
    if (rc != LORY_OK) return rc;
    // Every value the kernels read from the scratch is written earlier in the same call, so
    // nothing has to be cleared between calls.
    return dense_ffn_fwd(m, X, Wbar, Y, ws, st);
}

size_t dense_workspace_bytes(const Dims &m)
{
    if (gemm_path(m)) return bf16_dense_workspace_bytes(m);
    const SkinnyPlan pl = (m.dtype == LORY_F32) ? skinny_plan<float>(m) : skinny_plan<__hip_bfloat16>(m);
    return align_up(sizeof(float) * (pl.part1 + pl.part2), 256);
}

int dense_ffn_fwd(const Dims &m, const void *X, const void *Wbar, void *Y, void *ws, hipStream_t st)
{
    if (gemm_path(m)) return bf16_dense_ffn_fwd(m, X, Wbar, Y, ws, st);
    if (m.dtype == LORY_F32) return skinny_ffn<float>(m, (const float *)X, (const float *)Wbar, (float *)Y, ws, st);
    return skinny_ffn<__hip_bfloat16>(m, (const __hip_bfloat16 *)X, (const __hip_bfloat16 *)Wbar,
                                      (__hip_bfloat16 *)Y, ws, st);
}

}  // namespace lory
