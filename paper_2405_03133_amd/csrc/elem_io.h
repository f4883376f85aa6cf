// Element loads and stores shared by the HBM-bound kernels (routing, decode):
// 16 bytes per lane, widened to fp32 on the way in; bf16 stores round to nearest
// even (NaN stays NaN).
#pragma once

#include <hip/hip_bf16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lory {

template <typename T> struct Elem;

template <> struct Elem<float> {
    static constexpr int n = 4;    // elements of one 16-byte load
    static constexpr int vec = 4;
    __device__ static void load(const float *p, float (&v)[4])
    {
        const float4 q = *reinterpret_cast<const float4 *>(p);
        v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
    }
    __device__ static float one(const float *p) { return *p; }
    __device__ static void store(float *p, float v) { *p = v; }
};

template <> struct Elem<__hip_bfloat16> {
    static constexpr int n = 8;
    static constexpr int vec = 8;
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
    __device__ static void store(__hip_bfloat16 *p, float f)
    {
        const uint32_t u = __float_as_uint(f);
        uint16_t h;
        if ((u & 0x7fffffffu) > 0x7f800000u)
            h = (uint16_t)((u >> 16) | 0x40u);
        else
            h = (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
        *reinterpret_cast<uint16_t *>(p) = h;
    }
};

}  // namespace lory
