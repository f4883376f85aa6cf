// Causal segment routing on gfx950 (paper Section 3.1, Eq. 2; Algorithm 1):
// segment mean -> linear router -> softmax -> shift by one segment, with the
// first segment of every sequence routed on its own mean.
//
// One workgroup per segment.  The pass is HBM-bound (it reads X once); the
// mean, the logits and the softmax are all fp32 and every reduction has a
// fixed order, so results are deterministic.
#include "lory_internal.h"

#include <hip/hip_bf16.h>

namespace lory {

namespace {

constexpr int kRouteThreads = 1024;   // 16 wavefronts
constexpr int kColThreads = 256;      // threads along the hidden dimension
constexpr int kRowGroups = kRouteThreads / kColThreads;
constexpr int kMaxE = 64;

template <typename T> struct Vec;
template <> struct Vec<float> {
    static constexpr int n = 4;
    __device__ static void load(const float *p, float (&v)[4])
    {
        const float4 q = *reinterpret_cast<const float4 *>(p);
        v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
    }
    __device__ static float one(const float *p) { return *p; }
};
template <> struct Vec<__hip_bfloat16> {
    static constexpr int n = 8;
    __device__ static void load(const __hip_bfloat16 *p, float (&v)[8])
    {
        const uint4 q = *reinterpret_cast<const uint4 *>(p);
        const uint32_t r[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(r[i] << 16);
            v[2 * i + 1] = __uint_as_float(r[i] & 0xffff0000u);
        }
    }
    __device__ static float one(const __hip_bfloat16 *p)
    {
        return __uint_as_float(((uint32_t) * reinterpret_cast<const uint16_t *>(p)) << 16);
    }
};

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

    // ---- logits z[e] = sum_j hbar[j] * R[j][e]; thread = (e, one of 16 j-groups)
    {
        const int e = tid % 64;
        const int jg = tid / 64;
        float acc = 0.f;
        if (e < E) {
            int j = jg;
            for (; j + 7 * 16 < d; j += 8 * 16) {  // eight loads in flight, added in order
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

    // ---- softmax over the E experts by the first wavefront, then the shifted store
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
        const float prob = p / denom;
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
    {
        const int e = tid % 64, jg = tid / 64;
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
        const float pexp = (tid < E) ? expf(z - zmax) : 0.f;
        float denom = pexp;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) denom += __shfl_xor(denom, off, 64);
        if (tid < E) w[(size_t)b * E + tid] = pexp / denom;
    }
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
    if (m.dtype == LORY_F32) {
        if (m.d % Vec<float>::n == 0) return launch_route<float, true>(m, X, R, w, hbar, seg_len, st);
        return launch_route<float, false>(m, X, R, w, hbar, seg_len, st);
    }
    if (m.d % Vec<__hip_bfloat16>::n == 0) return launch_route<__hip_bfloat16, true>(m, X, R, w, hbar, seg_len, st);
    return launch_route<__hip_bfloat16, false>(m, X, R, w, hbar, seg_len, st);
}

}  // namespace lory
