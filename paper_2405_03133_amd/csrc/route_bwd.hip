// Backward of the causal segment routing on gfx950 (chain rule through paper
// Section 3.1 / Eq. 2; stop gradient on the first segment as in Algorithm 1).
//
// Forward: e[b,j] = softmax(hbar[b,j] R), w[b,0] = sg(e[b,0]), w[b,k] = e[b,k-1].
// Given dw (gradient with respect to the routing weights w of every segment):
//   de[b,j]   = dw[b,j+1] for j < N-1, 0 for the last segment of a sequence
//               (dw[b,0] is dropped: that use of e[b,0] sits behind the stop gradient)
//   dz[b,j]   = e[b,j] (.) (de[b,j] - <e[b,j], de[b,j]>)          softmax Jacobian
//   dR        = sum over segments of hbar[b,j]^T dz[b,j]
//   dhbar     = dz R^T,  dX[b, jT+t, :] += dhbar[b,j,:] / T        mean broadcast
// e[b,j] is read back from the forward's output as w[b,j+1]; the last segment's
// e is never needed because its dz is zero.
//
// Two kernels, both with fixed summation orders (bit-reproducible):
//   route_bwd_dx_kernel: HBM-bound read-modify-write of dX, grid (segments, row blocks)
//   route_bwd_dr_kernel: tiny [d, S] x [S, E] product, one workgroup per 16 rows of R
#include "lory_internal.h"

#include <hip/hip_bf16.h>

namespace lory {

namespace {

constexpr int kDxThreads = 256;
constexpr int kDrThreads = 1024;  // 64 experts x 16 rows of R
constexpr int kDrRows = 16;
constexpr int kDrChunk = 64;      // segments whose dz sit in LDS at a time

__device__ __forceinline__ float bf16_to_f32(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    const uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // NaN stays NaN
    return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

__device__ __forceinline__ float load_elem(const float *p) { return *p; }
__device__ __forceinline__ float load_elem(const __hip_bfloat16 *p)
{
    return bf16_to_f32(*reinterpret_cast<const uint16_t *>(p));
}

// <dz, one row of R>: 16-byte loads when the row length allows it.
__device__ __forceinline__ float dot_row(const float *__restrict__ row, const float *dz, int E)
{
    float acc = 0.f;
    if (E % 4 == 0) {
        for (int e = 0; e < E; e += 4) {
            const float4 v = *reinterpret_cast<const float4 *>(row + e);
            acc += dz[e] * v.x + dz[e + 1] * v.y + dz[e + 2] * v.z + dz[e + 3] * v.w;
        }
    } else {
        for (int e = 0; e < E; ++e) acc += dz[e] * row[e];
    }
    return acc;
}
__device__ __forceinline__ float dot_row(const __hip_bfloat16 *__restrict__ row, const float *dz, int E)
{
    float acc = 0.f;
    if (E % 8 == 0) {
        for (int e = 0; e < E; e += 8) {
            const uint4 q = *reinterpret_cast<const uint4 *>(row + e);
            const uint32_t r[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
            for (int i = 0; i < 4; ++i)
                acc += dz[e + 2 * i] * __uint_as_float(r[i] << 16) +
                       dz[e + 2 * i + 1] * __uint_as_float(r[i] & 0xffff0000u);
        }
    } else {
        for (int e = 0; e < E; ++e) acc += dz[e] * load_elem(row + e);
    }
    return acc;
}

// dz of segment s = b*N + j (j < N-1) for lane = expert; every lane of the wavefront takes part.
__device__ __forceinline__ float softmax_jacobian_row(const float *__restrict__ w, const float *__restrict__ dw,
                                                      int s, int E, int lane)
{
    float e = 0.f, de = 0.f;
    if (lane < E) {
        e = w[(size_t)(s + 1) * E + lane];
        de = dw[(size_t)(s + 1) * E + lane];
    }
    float inner = e * de;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) inner += __shfl_xor(inner, off, 64);
    return e * (de - inner);
}

// grid = (S, row blocks); block = 256 threads; LDS = 64 floats.
// Adds dhbar[s, :] / T to rows [rb * rows_per, ...) of segment s of dX.
template <typename T>
__global__ __launch_bounds__(kDxThreads) void route_bwd_dx_kernel(const T *__restrict__ R,
                                                                  const float *__restrict__ w,
                                                                  const float *__restrict__ dw,
                                                                  T *__restrict__ dX, int Tseg, int d,
                                                                  int E, int N, int rows_per)
{
    constexpr int VEC = 16 / (int)sizeof(T);  // elements per 16-byte access
    __shared__ float dz[64];
    const int s = blockIdx.x;
    if (s % N == N - 1) return;  // nothing routes on the last segment of a sequence
    const int tid = threadIdx.x;
    if (tid < 64) dz[tid] = softmax_jacobian_row(w, dw, s, E, tid);
    __syncthreads();

    const int t0 = blockIdx.y * rows_per;
    const int t1 = (t0 + rows_per < Tseg) ? (t0 + rows_per) : Tseg;
    const float invT = 1.0f / (float)Tseg;
    T *Xs = dX + (size_t)s * Tseg * d;

    if (d % VEC == 0) {
        for (int c = tid * VEC; c < d; c += kDxThreads * VEC) {
            float dh[VEC];
#pragma unroll
            for (int i = 0; i < VEC; ++i) dh[i] = dot_row(R + (size_t)(c + i) * E, dz, E) * invT;
            auto update = [&](uint4 q) {
                if constexpr (sizeof(T) == 4) {
                    q.x = __float_as_uint(__uint_as_float(q.x) + dh[0]);
                    q.y = __float_as_uint(__uint_as_float(q.y) + dh[1]);
                    q.z = __float_as_uint(__uint_as_float(q.z) + dh[2]);
                    q.w = __float_as_uint(__uint_as_float(q.w) + dh[3]);
                    return q;
                } else {
                    uint32_t r[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float lo = __uint_as_float(r[i] << 16) + dh[2 * i];
                        const float hi = __uint_as_float(r[i] & 0xffff0000u) + dh[2 * i + 1];
                        r[i] = (uint32_t)f32_to_bf16_rne(lo) | ((uint32_t)f32_to_bf16_rne(hi) << 16);
                    }
                    return make_uint4(r[0], r[1], r[2], r[3]);
                }
            };
            int t = t0;
            for (; t + 4 <= t1; t += 4) {  // four rows in flight
                uint4 q[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) q[u] = *reinterpret_cast<const uint4 *>(Xs + (size_t)(t + u) * d + c);
#pragma unroll
                for (int u = 0; u < 4; ++u) *reinterpret_cast<uint4 *>(Xs + (size_t)(t + u) * d + c) = update(q[u]);
            }
            for (; t < t1; ++t) {
                T *p = Xs + (size_t)t * d + c;
                *reinterpret_cast<uint4 *>(p) = update(*reinterpret_cast<const uint4 *>(p));
            }
        }
    } else {
        for (int c = tid; c < d; c += kDxThreads) {
            const float dh = dot_row(R + (size_t)c * E, dz, E) * invT;
            for (int t = t0; t < t1; ++t) {
                T *p = Xs + (size_t)t * d + c;
                if constexpr (sizeof(T) == 4) {
                    *p += dh;
                } else {
                    uint16_t *q = reinterpret_cast<uint16_t *>(p);
                    *q = f32_to_bf16_rne(bf16_to_f32(*q) + dh);
                }
            }
        }
    }
}

// grid = ceil(d / 16); block = 1024 threads: thread (expert = tid % 64, row = tid / 64).
// dR[c, e] (+)= sum over s in ascending order of hbar[s, c] * dz[s, e].
__global__ __launch_bounds__(kDrThreads) void route_bwd_dr_kernel(const float *__restrict__ hbar,
                                                                  const float *__restrict__ w,
                                                                  const float *__restrict__ dw,
                                                                  float *__restrict__ dR, int S, int d, int E,
                                                                  int N, int accumulate)
{
    __shared__ float dz[kDrChunk][64];
    const int tid = threadIdx.x;
    const int e = tid & 63, wave = tid >> 6;
    const int c = blockIdx.x * kDrRows + wave;
    float acc = 0.f;
    for (int s0 = 0; s0 < S; s0 += kDrChunk) {
        // 16 wavefronts, 4 segments each
#pragma unroll
        for (int i = 0; i < kDrChunk / 16; ++i) {
            const int sl = wave * (kDrChunk / 16) + i;
            const int s = s0 + sl;
            float v = 0.f;
            if (s < S && (s % N) != N - 1) v = softmax_jacobian_row(w, dw, s, E, e);
            dz[sl][e] = v;
        }
        __syncthreads();
        if (c < d) {
            const int n = (S - s0 < kDrChunk) ? (S - s0) : kDrChunk;
            for (int sl = 0; sl < n; ++sl) acc += hbar[(size_t)(s0 + sl) * d + c] * dz[sl][e];
        }
        __syncthreads();
    }
    if (c < d && e < E) {
        float *dst = dR + (size_t)c * E + e;
        *dst = accumulate ? (*dst + acc) : acc;
    }
}

template <typename T>
int launch_route_bwd(const Dims &m, const void *R, const float *w, const float *hbar, const float *dw,
                     void *dX, float *dR, int accumulate, hipStream_t st)
{
    // enough row blocks to give every CU a few workgroups, at least 8 rows each
    int rb = (1024 + m.S - 1) / m.S;
    if (rb > m.T / 8) rb = m.T / 8;
    if (rb < 1) rb = 1;
    const int rows_per = (m.T + rb - 1) / rb;
    rb = (m.T + rows_per - 1) / rows_per;
    hipLaunchKernelGGL((route_bwd_dx_kernel<T>), dim3(m.S, rb), dim3(kDxThreads), 0, st, (const T *)R, w, dw,
                       (T *)dX, m.T, m.d, m.E, m.N, rows_per);
    if (hipGetLastError() != hipSuccess) return LORY_ERR_DEVICE;
    hipLaunchKernelGGL(route_bwd_dr_kernel, dim3((m.d + kDrRows - 1) / kDrRows), dim3(kDrThreads), 0, st, hbar,
                       w, dw, dR, m.S, m.d, m.E, m.N, accumulate);
    return launch_status();
}

}  // namespace

int route_bwd_launch(const Dims &m, const void *R, const float *w, const float *hbar, const float *dw,
                     void *dX, float *dR, int accumulate, hipStream_t st)
{
    if (m.dtype == LORY_F32) return launch_route_bwd<float>(m, R, w, hbar, dw, dX, dR, accumulate, st);
    return launch_route_bwd<__hip_bfloat16>(m, R, w, hbar, dw, dX, dR, accumulate, st);
}

}  // namespace lory
