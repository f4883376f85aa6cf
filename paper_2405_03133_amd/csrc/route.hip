// Causal segment routing on gfx950 (paper Section 3.1, Eq. 2; Algorithm 1):
// segment mean -> linear router -> softmax -> shift by one segment, with the
// first segment of every sequence routed on its own mean.
//
// One workgroup per segment, or (training shapes that return the segment
// means) a first pass over (segment, column block) workgroups for the means
// and a second one for the router.  The pass is HBM-bound (it reads X once);
// the mean, the logits and the softmax are all fp32 and every reduction has a
// fixed order, so results are deterministic.
#include "lory_internal.h"

#include "elem_io.h"

namespace lory {

namespace {

template <typename T> using Vec = Elem<T>;

constexpr int kRouteThreads = 1024;   // 16 wavefronts
constexpr int kColThreads = 256;      // threads along the hidden dimension
constexpr int kRowGroups = kRouteThreads / kColThreads;
constexpr int kMaxE = 64;

// Router of one segment (Section 3: a linear layer, then a softmax over the E experts): logits
// z[e] = sum_j hbar[j] * R[j][e] with thread = (e, one of 16 j-groups), eight loads in flight and
// added in order; the 16 partial sums are added in group order by the first wavefront, which then
// takes the max-subtracted softmax with wavefront reductions.  hbar [d] and zpart [16][64] are in
// LDS; all 1024 threads call this; lanes tid < E of the first wavefront return the probability of
// expert tid, everyone else 0.
template <typename T>
__device__ __forceinline__ float router_softmax(const float *hbar, float *zpart, const T *__restrict__ R, int d,
                                                int E, int tid)
{
    {
        const int e = tid % 64;
        const int jg = tid / 64;
        float acc = 0.f;
        if (e < E) {
            int j = jg;
            for (; j + 7 * 16 < d; j += 8 * 16) {
                float r[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) r[i] = Vec<T>::one(R + (size_t)(j + 16 * i) * E + e);
#pragma unroll
                for (int i = 0; i < 8; ++i) acc += hbar[j + 16 * i] * r[i];
            }
            for (; j < d; j += 16) acc += hbar[j] * Vec<T>::one(R + (size_t)j * E + e);
        }
        zpart[jg * 64 + e] = acc;
    }
    __syncthreads();
    float prob = 0.f;
    if (tid < 64) {
        float z = -INFINITY;
        if (tid < E) {
            z = 0.f;
#pragma unroll
            for (int g = 0; g < 16; ++g) z += zpart[g * 64 + tid];
        }
        float zmax = z;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) zmax = fmaxf(zmax, __shfl_xor(zmax, off, 64));
        const float p = (tid < E) ? expf(z - zmax) : 0.f;
        float denom = p;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) denom += __shfl_xor(denom, off, 64);
        prob = p / denom;
    }
    return prob;
}

// grid = S workgroups, block = 1024 threads, dynamic LDS =
// (d + kRowGroups * kColThreads * VEC + 16 * 64) floats.
template <typename T, bool VECTOR>
__global__ __launch_bounds__(kRouteThreads) void route_kernel(const T *__restrict__ X,
                                                              const T *__restrict__ R,
                                                              float *__restrict__ w,
                                                              float *__restrict__ hbar_out,
                                                              const int32_t *__restrict__ seg_len,
                                                              int Tseg, int d, int E, int N)
{
    constexpr int VEC = VECTOR ? Vec<T>::n : 1;
    extern __shared__ float lds[];
    float *hbar = lds;                                   // [d]
    float *part = lds + d;                               // [kRowGroups][kColThreads*VEC]
    float *zpart = part + kRowGroups * kColThreads * VEC; // [16][64]

    const int s = blockIdx.x;
    const int k = s % N;
    const int tid = threadIdx.x;
    const int tx = tid % kColThreads;
    const int ty = tid / kColThreads;
    const T *Xs = X + (size_t)s * Tseg * d;
    // rows that enter the mean: all Tseg, or (prompts of different lengths, padded to Tseg rows)
    // the first seg_len[s] of them, clamped to 1 .. Tseg
    int rows = Tseg;
    if (seg_len) {
        rows = seg_len[s];
        rows = rows < 1 ? 1 : (rows > Tseg ? Tseg : rows);
    }
    const float invT = 1.0f / (float)rows;

    // ---- segment mean, a chunk of kColThreads*VEC columns at a time
    for (int c0 = 0; c0 < d; c0 += kColThreads * VEC) {
        const int c = c0 + tx * VEC;
        float acc[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
        if (c < d) {
            int t = ty;
            for (; t + 3 * kRowGroups < rows; t += 4 * kRowGroups) {  // four rows in flight, added in row order
                float v[4][VEC];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if constexpr (VECTOR) {
                        Vec<T>::load(Xs + (size_t)(t + u * kRowGroups) * d + c, v[u]);
                    } else {
                        v[u][0] = Vec<T>::one(Xs + (size_t)(t + u * kRowGroups) * d + c);
                    }
                }
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int i = 0; i < VEC; ++i) acc[i] += v[u][i];
            }
            for (; t < rows; t += kRowGroups) {
                float v[VEC];
                if constexpr (VECTOR) {
                    Vec<T>::load(Xs + (size_t)t * d + c, v);
                } else {
                    v[0] = Vec<T>::one(Xs + (size_t)t * d + c);
                }
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[i] += v[i];
            }
        }
#pragma unroll
        for (int i = 0; i < VEC; ++i) part[(ty * kColThreads + tx) * VEC + i] = acc[i];
        __syncthreads();
        if (ty == 0 && c < d) {
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                float sum = 0.f;
#pragma unroll
                for (int g = 0; g < kRowGroups; ++g) sum += part[(g * kColThreads + tx) * VEC + i];
                const float mean = sum * invT;
                hbar[c + i] = mean;
                if (hbar_out) hbar_out[(size_t)s * d + c + i] = mean;
            }
        }
        __syncthreads();
    }

    const float prob = router_softmax<T>(hbar, zpart, R, d, E, tid);
    if (tid < 64) {
        if (tid < E) {
            // Segment k routes segment k+1; segment 0 also routes itself.
            if (k == 0) w[(size_t)s * E + tid] = prob;
            if (k + 1 < N) w[(size_t)(s + 1) * E + tid] = prob;
        }
    }
}

// ---- routing on the mean of a whole (long) prompt, two stages so that a handful of sequences
// still fills the chip.  Stage 1: grid (sequences, row chunks), column sums of the chunk's rows
// (only rows below the sequence's prompt length) into part[b][chunk][d].  Stage 2: one workgroup
// per sequence adds the chunks in order, divides by the length, and runs the logits and the
// softmax exactly like route_kernel.
constexpr int kPromptChunkRows = 64;

template <typename T>
__global__ __launch_bounds__(256) void prompt_sum_kernel(const T *__restrict__ X, const int32_t *__restrict__ len,
                                                         float *__restrict__ part, int L, int d, int chunks)
{
    constexpr int VEC = Vec<T>::n;
    const int b = blockIdx.x, ch = blockIdx.y;
    int rows = len ? len[b] : L;
    rows = rows < 1 ? 1 : (rows > L ? L : rows);
    const int r0 = ch * kPromptChunkRows;
    const int r1 = (r0 + kPromptChunkRows < rows) ? (r0 + kPromptChunkRows) : rows;
    const T *Xb = X + (size_t)b * L * d;
    float *dst = part + ((size_t)b * chunks + ch) * d;
    if (d % VEC == 0) {
        for (int c = threadIdx.x * VEC; c < d; c += 256 * VEC) {
            float acc[VEC];
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
            for (int t = r0; t < r1; ++t) {
                float v[VEC];
                Vec<T>::load(Xb + (size_t)t * d + c, v);
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[i] += v[i];
            }
#pragma unroll
            for (int i = 0; i < VEC; ++i) dst[c + i] = acc[i];
        }
    } else {
        for (int c = threadIdx.x; c < d; c += 256) {
            float acc = 0.f;
            for (int t = r0; t < r1; ++t) acc += Vec<T>::one(Xb + (size_t)t * d + c);
            dst[c] = acc;
        }
    }
}

// grid = sequences, block = 1024, dynamic LDS = (d + 16 * 64) floats.
template <typename T>
__global__ __launch_bounds__(kRouteThreads) void prompt_finish_kernel(const float *__restrict__ part,
                                                                      const int32_t *__restrict__ len,
                                                                      const T *__restrict__ R,
                                                                      float *__restrict__ w, int L, int d, int E,
                                                                      int chunks)
{
    extern __shared__ float lds[];
    float *hbar = lds;         // [d]
    float *zpart = lds + d;    // [16][64]
    const int b = blockIdx.x, tid = threadIdx.x;
    int rows = len ? len[b] : L;
    rows = rows < 1 ? 1 : (rows > L ? L : rows);
    const int used = (rows + kPromptChunkRows - 1) / kPromptChunkRows;
    const float inv = 1.0f / (float)rows;
    for (int c = tid; c < d; c += kRouteThreads) {
        const float *src = part + (size_t)b * chunks * d + c;
        float sum = 0.f;
        int ch = 0;
        for (; ch + 8 <= used; ch += 8) {  // loads overlap, adds stay in chunk order
            float v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = src[(size_t)(ch + i) * d];
#pragma unroll
            for (int i = 0; i < 8; ++i) sum += v[i];
        }
        for (; ch < used; ++ch) sum += src[(size_t)ch * d];
        hbar[c] = sum * inv;
    }
    __syncthreads();
    const float prob = router_softmax<T>(hbar, zpart, R, d, E, tid);
    if (tid < E) w[(size_t)b * E + tid] = prob;
}

template <typename T>
int launch_prompt_route(const Dims &m, const void *X, const int32_t *len, const void *R, float *w, float *scratch,
                        hipStream_t st)
{
    const int chunks = (m.L + kPromptChunkRows - 1) / kPromptChunkRows;
    hipLaunchKernelGGL((prompt_sum_kernel<T>), dim3(m.B, chunks), dim3(256), 0, st, (const T *)X, len, scratch, m.L,
                       m.d, chunks);
    if (hipGetLastError() != hipSuccess) return LORY_ERR_DEVICE;
    const size_t lds = sizeof(float) * ((size_t)m.d + 16 * 64);
    if (lds > 48 * 1024) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&prompt_finish_kernel<T>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return LORY_ERR_DEVICE;
    }
    hipLaunchKernelGGL((prompt_finish_kernel<T>), dim3(m.B), dim3(kRouteThreads), lds, st, scratch, len,
                       (const T *)R, w, m.L, m.d, m.E, chunks);
    return launch_status();
}

size_t route_lds_bytes(int d, int vec)
{
    return sizeof(float) * ((size_t)d + (size_t)kRowGroups * kColThreads * vec + 16 * 64);
}

// ---- training shapes with hbar requested: two stages, so that a few dozen segments still fill the
// chip.  Stage 1: grid (segments, column blocks): every workgroup takes the mean of its 256 (bf16;
// 128 for fp32) columns over all T rows, eight rows per thread in flight, and writes it to hbar.
// Stage 2: one workgroup per segment reads its hbar row back and routes.
constexpr int kMeanRowGroups = 8;

template <typename T>
__global__ __launch_bounds__(256) void route_mean_kernel(const T *__restrict__ X, float *__restrict__ hbar_out,
                                                         int Tseg, int d)
{
    constexpr int VEC = Vec<T>::n;
    constexpr int COLS = 256 / kMeanRowGroups;   // column threads
    __shared__ float part[kMeanRowGroups][COLS * VEC];
    const int s = blockIdx.x;
    const int tx = threadIdx.x % COLS, ty = threadIdx.x / COLS;
    const int c = (blockIdx.y * COLS + tx) * VEC;
    const T *Xs = X + (size_t)s * Tseg * d;
    float acc[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
    if (c < d) {
        int t = ty;
        for (; t + 7 * kMeanRowGroups < Tseg; t += 8 * kMeanRowGroups) {  // eight rows in flight, added in row order
            float v[8][VEC];
#pragma unroll
            for (int u = 0; u < 8; ++u) Vec<T>::load(Xs + (size_t)(t + u * kMeanRowGroups) * d + c, v[u]);
#pragma unroll
            for (int u = 0; u < 8; ++u)
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[i] += v[u][i];
        }
        for (; t < Tseg; t += kMeanRowGroups) {
            float v[VEC];
            Vec<T>::load(Xs + (size_t)t * d + c, v);
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] += v[i];
        }
    }
#pragma unroll
    for (int i = 0; i < VEC; ++i) part[ty][tx * VEC + i] = acc[i];
    __syncthreads();
    if (ty == 0 && c < d) {
        const float invT = 1.0f / (float)Tseg;
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
            float sum = 0.f;
#pragma unroll
            for (int g = 0; g < kMeanRowGroups; ++g) sum += part[g][tx * VEC + i];
            hbar_out[(size_t)s * d + c + i] = sum * invT;
        }
    }
}

// grid = segments, block = 1024, dynamic LDS = (d + 16 * 64) floats.
template <typename T>
__global__ __launch_bounds__(kRouteThreads) void route_finish_kernel(const float *__restrict__ hbar_in,
                                                                     const T *__restrict__ R,
                                                                     float *__restrict__ w, int d, int E, int N)
{
    extern __shared__ float lds[];
    float *hbar = lds;         // [d]
    float *zpart = lds + d;    // [16][64]
    const int s = blockIdx.x, k = s % N, tid = threadIdx.x;
    for (int c = tid; c < d; c += kRouteThreads) hbar[c] = hbar_in[(size_t)s * d + c];
    __syncthreads();
    const float prob = router_softmax<T>(hbar, zpart, R, d, E, tid);
    if (tid < E) {
        // Segment k routes segment k+1; segment 0 also routes itself.
        if (k == 0) w[(size_t)s * E + tid] = prob;
        if (k + 1 < N) w[(size_t)(s + 1) * E + tid] = prob;
    }
}

template <typename T>
int launch_route_two_stage(const Dims &m, const void *X, const void *R, float *w, float *hbar, hipStream_t st)
{
    constexpr int cols = (256 / kMeanRowGroups) * Vec<T>::n;
    hipLaunchKernelGGL((route_mean_kernel<T>), dim3(m.S, (m.d + cols - 1) / cols), dim3(256), 0, st, (const T *)X,
                       hbar, m.T, m.d);
    if (hipGetLastError() != hipSuccess) return LORY_ERR_DEVICE;
    const size_t lds = sizeof(float) * ((size_t)m.d + 16 * 64);
    if (lds > 48 * 1024) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&route_finish_kernel<T>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return LORY_ERR_DEVICE;
    }
    hipLaunchKernelGGL((route_finish_kernel<T>), dim3(m.S), dim3(kRouteThreads), lds, st, hbar, (const T *)R, w, m.d,
                       m.E, m.N);
    return launch_status();
}

template <typename T, bool VECTOR>
int launch_route(const Dims &m, const void *X, const void *R, float *w, float *hbar, const int32_t *seg_len,
                 hipStream_t st)
{
    const size_t lds = route_lds_bytes(m.d, VECTOR ? Vec<T>::n : 1);
    if (lds > 48 * 1024) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&route_kernel<T, VECTOR>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return LORY_ERR_DEVICE;
    }
    hipLaunchKernelGGL((route_kernel<T, VECTOR>), dim3(m.S), dim3(kRouteThreads), lds, st,
                       (const T *)X, (const T *)R, w, hbar, seg_len, m.T, m.d, m.E, m.N);
    return launch_status();
}

}  // namespace

size_t prompt_route_scratch_bytes(const Dims &m)
{
    const size_t chunks = ((size_t)m.L + kPromptChunkRows - 1) / kPromptChunkRows;
    return sizeof(float) * (size_t)m.B * chunks * m.d;
}

// Routing weights of every sequence from the mean of its whole prompt (m.T == m.L).  `scratch`
// holds prompt_route_scratch_bytes(m) bytes.
int prompt_route_launch(const Dims &m, const void *X, const int32_t *len, const void *R, float *w, float *scratch,
                        hipStream_t st)
{
    if (m.dtype == LORY_F32) return launch_prompt_route<float>(m, X, len, R, w, scratch, st);
    return launch_prompt_route<__hip_bfloat16>(m, X, len, R, w, scratch, st);
}

int route_launch(const Dims &m, const void *X, const void *R, float *w, float *hbar, const int32_t *seg_len,
                 hipStream_t st)
{
    static_assert(kMaxE == 64, "logit stage assumes E <= 64");
    // The segment means double as the exchange buffer of the two-stage path; it pays when one
    // workgroup per segment would leave most of the chip idle.
    if (hbar && !seg_len && m.S < 512 && m.T >= 32) {
        if (m.dtype == LORY_F32 && m.d % Vec<float>::n == 0) return launch_route_two_stage<float>(m, X, R, w, hbar, st);
        if (m.dtype == LORY_BF16 && m.d % Vec<__hip_bfloat16>::n == 0)
            return launch_route_two_stage<__hip_bfloat16>(m, X, R, w, hbar, st);
    }
    if (m.dtype == LORY_F32) {
        if (m.d % Vec<float>::n == 0) return launch_route<float, true>(m, X, R, w, hbar, seg_len, st);
        return launch_route<float, false>(m, X, R, w, hbar, seg_len, st);
    }
    if (m.d % Vec<__hip_bfloat16>::n == 0) return launch_route<__hip_bfloat16, true>(m, X, R, w, hbar, seg_len, st);
    return launch_route<__hip_bfloat16, false>(m, X, R, w, hbar, seg_len, st);
}

}  // namespace lory
