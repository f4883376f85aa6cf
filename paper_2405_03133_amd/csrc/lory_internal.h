// Internal declarations shared by the translation units of liblory.so.
// Not part of the public ABI (that is include/lory.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "lory.h"

namespace lory {

// Derived sizes of a validated shape.
struct Dims {
    int B, L, T, d, dff, E;
    int N;         // segments per sequence
    int S;         // segments in total
    long tokens;   // B * L
    long D;        // d * d_ff, elements of one expert matrix
    int dtype;
};

inline Dims make_dims(const lory_shape &s)
{
    Dims m;
    m.B = s.B; m.L = s.L; m.T = s.T; m.d = s.d; m.dff = s.d_ff; m.E = s.E;
    m.N = s.L / s.T;
    m.S = s.B * m.N;
    m.tokens = (long)s.B * s.L;
    m.D = (long)s.d * s.d_ff;
    m.dtype = s.dtype;
    return m;
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Turns the last launch error into a status.
inline int launch_status()
{
    return hipGetLastError() == hipSuccess ? LORY_OK : LORY_ERR_DEVICE;
}

// ---- optional event timing per kernel class (profile.hip)
namespace prof {
enum Class { kRoute = 0, kMerge, kGemmGU, kSwigluFwd, kGemmDown, kGemmDA, kSwigluBwd, kGemmDX, kGemmDWGU, kGemmDWD, kScatter,
             kDwReduce, kRouteBwd, kDenseSkinny, kFusedGU, kFusedDown, kFusedDA, kFusedDX, kFusedDW,
             kNumClasses };
bool enabled();
int set_enabled(int on);
int read(lory_kernel_stat *out, int max_out, int *n_out);
// Brackets the launches issued during its lifetime with two events (only when enabled).
class Range {
public:
    Range(hipStream_t st, int cls, double flops, double bytes);
    ~Range();
    Range(const Range &) = delete;
    Range &operator=(const Range &) = delete;
private:
    hipStream_t st_;
    int idx_;
};
}  // namespace prof

// ---- routing (route.hip)
int route_launch(const Dims &m, const void *X, const void *R, float *w, float *hbar, const int32_t *seg_len,
                 hipStream_t st);

size_t prompt_route_scratch_bytes(const Dims &m);
int prompt_route_launch(const Dims &m, const void *X, const int32_t *len, const void *R, float *w, float *scratch,
                        hipStream_t st);

// ---- routing backward (route_bwd.hip)
int route_bwd_launch(const Dims &m, const void *R, const float *w, const float *hbar, const float *dw,
                     void *dX, float *dR, int accumulate, hipStream_t st);

// ---- fp32 path (ffn_f32.hip)
size_t f32_workspace_bytes(const Dims &m, int pass);
int f32_ffn_fwd(const Dims &m, const float *X, const float *w, const float *Wg, const float *Wu,
                const float *Wd, float *Y, float *G_save, float *U_save, void *ws, hipStream_t st);
int f32_ffn_bwd(const Dims &m, const float *X, const float *w, const float *Wg, const float *Wu,
                const float *Wd, const float *dY, const float *G_save, const float *U_save,
                float *dX, float *dWg, float *dWu, float *dWd, int accumulate, float *dw,
                void *ws, hipStream_t st);

int f32_merge_all(const Dims &m, const float *w, const float *Wg, const float *Wu, const float *Wd,
                  float *Wbar, hipStream_t st);

// ---- inference with prompt-only routing (infer.hip)
size_t dense_workspace_bytes(const Dims &m);
int dense_ffn_fwd(const Dims &m, const void *X, const void *Wbar, void *Y, void *ws, hipStream_t st);
size_t dense_static_scratch_limit();
int dense_ffn_fwd_static(const Dims &m, const void *X, const void *Wbar, void *Y, hipStream_t st);

// ---- bf16 path (ffn_bf16.hip)
int bf16_merge_all(const Dims &m, const float *w, const void *Wg, const void *Wu, const void *Wd,
                   void *Wbar, hipStream_t st);
size_t bf16_dense_workspace_bytes(const Dims &m);
int bf16_dense_ffn_fwd(const Dims &m, const void *X, const void *Wbar, void *Y, void *ws, hipStream_t st);
int set_slab_budget(size_t bytes);
int set_fused_mode(int mode);
size_t bf16_workspace_bytes(const Dims &m, int pass);
size_t bf16_merged_save_bytes(const Dims &m);
int bf16_ffn_fwd(const Dims &m, const void *X, const float *w, const void *Wg, const void *Wu,
                 const void *Wd, void *Y, void *G_save, void *U_save, void *Wbar_save, void *ws,
                 hipStream_t st);
int bf16_ffn_bwd(const Dims &m, const void *X, const float *w, const void *Wg, const void *Wu,
                 const void *Wd, const void *dY, const void *G_save, const void *U_save,
                 const void *Wbar_save, void *dX, void *dWg, void *dWu, void *dWd, int grad_dtype,
                 int accumulate, float *dw, void *ws, hipStream_t st);

}  // namespace lory
