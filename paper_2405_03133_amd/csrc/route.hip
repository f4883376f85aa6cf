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
            for (int t = ty; t < rows; t += kRowGroups) {
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
            for (int j = jg; j < d; j += 16) acc += hbar[j] * Vec<T>::one(R + (size_t)j * E + e);
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
