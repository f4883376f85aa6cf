// extern "C" entry points of liblory.so: argument validation, dispatch on the
// storage dtype, launch on the caller's stream.  See include/lory.h for the
// contract of every call.
#include "lory_internal.h"

namespace {

using lory::Dims;

int check_shape(const lory_shape *s)
{
    if (!s) return LORY_ERR_NULL;
    if (s->dtype != LORY_F32 && s->dtype != LORY_BF16) return LORY_ERR_DTYPE;
    if (s->B <= 0 || s->L <= 0 || s->T <= 0 || s->d <= 0 || s->d_ff <= 0 || s->E <= 0)
        return LORY_ERR_SHAPE;
    if (s->L % s->T != 0) return LORY_ERR_SHAPE;
    if (s->E > 64) return LORY_ERR_SHAPE;
    if (s->d > 16384) return LORY_ERR_SHAPE;  // the routing kernel keeps one mean vector in LDS
    if ((long)s->B * (s->L / s->T) > 65535) return LORY_ERR_SHAPE;  // segments index a grid dimension
    if (s->dtype == LORY_BF16) {
        if (s->d % 64 != 0 || s->d_ff % 64 != 0 || s->T % 64 != 0) return LORY_ERR_SHAPE;
    }
    return LORY_OK;
}

// The inference entry points treat every sequence as one segment (T == L) of any length.
int check_shape_infer(const lory_shape *s)
{
    if (!s) return LORY_ERR_NULL;
    if (s->dtype != LORY_F32 && s->dtype != LORY_BF16) return LORY_ERR_DTYPE;
    if (s->B <= 0 || s->L <= 0 || s->T <= 0 || s->d <= 0 || s->d_ff <= 0 || s->E <= 0)
        return LORY_ERR_SHAPE;
    if (s->T != s->L) return LORY_ERR_SHAPE;
    if (s->E > 64 || s->d > 16384 || s->B > 65535) return LORY_ERR_SHAPE;
    if (s->dtype == LORY_BF16 && (s->d % 64 != 0 || s->d_ff % 64 != 0)) return LORY_ERR_SHAPE;
    return LORY_OK;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

extern "C" {

const char *lory_status_string(int status)
{
    switch (status) {
    case LORY_OK: return "ok";
    case LORY_ERR_NULL: return "required pointer is NULL";
    case LORY_ERR_SHAPE: return "invalid shape (dimension <= 0, L % T != 0, or granularity rule violated)";
    case LORY_ERR_DTYPE: return "unknown or unsupported dtype";
    case LORY_ERR_ALIGN: return "pointer is not 16-byte aligned";
    case LORY_ERR_WORKSPACE: return "workspace too small";
    case LORY_ERR_DEVICE: return "HIP call or kernel launch failed";
    default: return "unknown status";
    }
}

const char *lory_version(void) { return "0.1"; }

int lory_set_slab_budget(size_t bytes) { return lory::set_slab_budget(bytes); }

int lory_set_fused_merge(int mode) { return lory::set_fused_mode(mode); }

int lory_profile_enable(int on) { return lory::prof::set_enabled(on); }

int lory_profile_read(lory_kernel_stat *out, int max_out, int *n_out)
{
    if (!out || !n_out) return LORY_ERR_NULL;
    if (max_out <= 0) return LORY_ERR_SHAPE;
    return lory::prof::read(out, max_out, n_out);
}

int lory_merged_save_bytes(const lory_shape *shape, size_t *bytes_out)
{
    if (!bytes_out) return LORY_ERR_NULL;
    const int rc = check_shape(shape);
    if (rc != LORY_OK) return rc;
    const Dims m = lory::make_dims(*shape);
    *bytes_out = (m.dtype == LORY_BF16) ? lory::bf16_merged_save_bytes(m) : 0;
    return LORY_OK;
}

int lory_workspace_bytes(const lory_shape *shape, int pass, size_t *bytes_out)
{
    if (!bytes_out) return LORY_ERR_NULL;
    if (pass == LORY_PASS_DENSE) {
        const int rci = check_shape_infer(shape);
        if (rci != LORY_OK) return rci;
        *bytes_out = lory::align_up(lory::dense_workspace_bytes(lory::make_dims(*shape)), 256);
        return LORY_OK;
    }
    const int rc = check_shape(shape);
    if (rc != LORY_OK) return rc;
    if (pass != LORY_PASS_FWD && pass != LORY_PASS_BWD) return LORY_ERR_SHAPE;
    const Dims m = lory::make_dims(*shape);
    const size_t n = (m.dtype == LORY_F32) ? lory::f32_workspace_bytes(m, pass)
                                           : lory::bf16_workspace_bytes(m, pass);
    *bytes_out = lory::align_up(n, 256);
    return LORY_OK;
}

int lory_route(const lory_shape *shape, const void *X, const void *R, float *w, float *hbar_opt,
               void *stream)
{
    const int rc = check_shape(shape);
    if (rc != LORY_OK) return rc;
    if (!X || !R || !w) return LORY_ERR_NULL;
    if (!aligned16(X) || !aligned16(R) || !aligned16(w) || !aligned16(hbar_opt)) return LORY_ERR_ALIGN;
    const Dims m = lory::make_dims(*shape);
    const double esz = (m.dtype == LORY_F32) ? 4.0 : 2.0;
    lory::prof::Range r((hipStream_t)stream, lory::prof::kRoute, 2.0 * m.S * m.d * m.E + (double)m.tokens * m.d,
                        esz * ((double)m.tokens * m.d + (double)m.d * m.E) + 4.0 * m.S * m.E);
    return lory::route_launch(m, X, R, w, hbar_opt, nullptr, (hipStream_t)stream);
}

int lory_route_bwd(const lory_shape *shape, const void *R, const float *w, const float *hbar,
                   const float *dw, void *dX, float *dR, int accumulate_dR, void *stream)
{
    const int rc = check_shape(shape);
    if (rc != LORY_OK) return rc;
    if (!R || !w || !hbar || !dw || !dX || !dR) return LORY_ERR_NULL;
    if (accumulate_dR != 0 && accumulate_dR != 1) return LORY_ERR_SHAPE;
    if (!aligned16(R) || !aligned16(w) || !aligned16(hbar) || !aligned16(dw) || !aligned16(dX) ||
        !aligned16(dR))
        return LORY_ERR_ALIGN;
    const Dims m = lory::make_dims(*shape);
    const double esz = (m.dtype == LORY_F32) ? 4.0 : 2.0;
    // every segment but the last of each sequence has its rows of dX read and written
    const double rows = (double)m.B * (m.N - 1) * m.T;
    lory::prof::Range r((hipStream_t)stream, lory::prof::kRouteBwd,
                        4.0 * m.S * m.d * m.E + rows * m.d,
                        2.0 * esz * rows * m.d + 4.0 * ((double)m.S * m.d + (double)m.d * m.E));
    return lory::route_bwd_launch(m, R, w, hbar, dw, dX, dR, accumulate_dR, (hipStream_t)stream);
}

int lory_prompt_merge(const lory_shape *shape, const void *X_prompt, const int32_t *prompt_len_opt,
                      const void *R, const void *Wg, const void *Wu, const void *Wd, float *w, void *Wbar,
                      void *stream)
{
    const int rc = check_shape_infer(shape);
    if (rc != LORY_OK) return rc;
    if (!X_prompt || !R || !Wg || !Wu || !Wd || !w || !Wbar) return LORY_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(prompt_len_opt) & 3u) != 0) return LORY_ERR_ALIGN;
    if (!aligned16(X_prompt) || !aligned16(R) || !aligned16(Wg) || !aligned16(Wu) || !aligned16(Wd) ||
        !aligned16(w) || !aligned16(Wbar))
        return LORY_ERR_ALIGN;
    const Dims m = lory::make_dims(*shape);
    hipStream_t st = (hipStream_t)stream;
    {
        const double esz = (m.dtype == LORY_F32) ? 4.0 : 2.0;
        lory::prof::Range r(st, lory::prof::kRoute, 2.0 * m.S * m.d * m.E + (double)m.tokens * m.d,
                            esz * ((double)m.tokens * m.d + (double)m.d * m.E) + 4.0 * m.S * m.E);
        // Long prompts of a few sequences: the mean is taken in two stages over many workgroups,
        // with the partial sums parked in Wbar, which the merges overwrite afterwards.
        const size_t esize = (m.dtype == LORY_F32) ? 4 : 2;
        const bool two_stage = m.L >= 256 && lory::prompt_route_scratch_bytes(m) <= (size_t)3 * m.B * m.D * esize;
        const int rr = two_stage ? lory::prompt_route_launch(m, X_prompt, prompt_len_opt, R, w, (float *)Wbar, st)
                                 : lory::route_launch(m, X_prompt, R, w, nullptr, prompt_len_opt, st);
        if (rr != LORY_OK) return rr;
    }
    if (m.dtype == LORY_F32)
        return lory::f32_merge_all(m, w, (const float *)Wg, (const float *)Wu, (const float *)Wd,
                                   (float *)Wbar, st);
    return lory::bf16_merge_all(m, w, Wg, Wu, Wd, Wbar, st);
}

int lory_dense_ffn_fwd(const lory_shape *shape, const void *X, const void *Wbar, void *Y,
                       void *workspace, size_t workspace_bytes, void *stream)
{
    const int rc = check_shape_infer(shape);
    if (rc != LORY_OK) return rc;
    if (!X || !Wbar || !Y || !workspace) return LORY_ERR_NULL;
    if (!aligned16(X) || !aligned16(Wbar) || !aligned16(Y) || !aligned16(workspace)) return LORY_ERR_ALIGN;
    const Dims m = lory::make_dims(*shape);
    if (workspace_bytes < lory::align_up(lory::dense_workspace_bytes(m), 256)) return LORY_ERR_WORKSPACE;
    return lory::dense_ffn_fwd(m, X, Wbar, Y, workspace, (hipStream_t)stream);
}

int lory_dense_ffn_fwd_static(const lory_shape *shape, const void *X, const void *Wbar, void *Y, void *stream)
{
    const int rc = check_shape_infer(shape);
    if (rc != LORY_OK) return rc;
    if (!X || !Wbar || !Y) return LORY_ERR_NULL;
    if (!aligned16(X) || !aligned16(Wbar) || !aligned16(Y)) return LORY_ERR_ALIGN;
    const Dims m = lory::make_dims(*shape);
    if (lory::align_up(lory::dense_workspace_bytes(m), 256) > lory::dense_static_scratch_limit())
        return LORY_ERR_WORKSPACE;
    return lory::dense_ffn_fwd_static(m, X, Wbar, Y, (hipStream_t)stream);
}

int lory_merged_ffn_fwd(const lory_shape *shape, const void *X, const float *w, const void *Wg,
                        const void *Wu, const void *Wd, void *Y, void *G_save, void *U_save,
                        void *Wbar_save, void *workspace, size_t workspace_bytes, void *stream)
{
    const int rc = check_shape(shape);
    if (rc != LORY_OK) return rc;
    if (!X || !w || !Wg || !Wu || !Wd || !Y || !workspace) return LORY_ERR_NULL;
    if ((G_save == nullptr) != (U_save == nullptr)) return LORY_ERR_NULL;
    if (!aligned16(X) || !aligned16(w) || !aligned16(Wg) || !aligned16(Wu) || !aligned16(Wd) ||
        !aligned16(Y) || !aligned16(G_save) || !aligned16(U_save) || !aligned16(Wbar_save) ||
        !aligned16(workspace))
        return LORY_ERR_ALIGN;
    if (Wbar_save) {
        size_t sb = 0;
        lory_merged_save_bytes(shape, &sb);
        if (sb == 0) return LORY_ERR_SHAPE;
    }
    size_t need = 0;
    lory_workspace_bytes(shape, LORY_PASS_FWD, &need);
    if (workspace_bytes < need) return LORY_ERR_WORKSPACE;
    const Dims m = lory::make_dims(*shape);
    hipStream_t st = (hipStream_t)stream;
    if (m.dtype == LORY_F32)
        return lory::f32_ffn_fwd(m, (const float *)X, w, (const float *)Wg, (const float *)Wu,
                                 (const float *)Wd, (float *)Y, (float *)G_save, (float *)U_save,
                                 workspace, st);
    return lory::bf16_ffn_fwd(m, X, w, Wg, Wu, Wd, Y, G_save, U_save, Wbar_save, workspace, st);
}

int lory_merged_ffn_bwd(const lory_shape *shape, const void *X, const float *w, const void *Wg,
                        const void *Wu, const void *Wd, const void *dY, const void *G_save,
                        const void *U_save, const void *Wbar_save, void *dX, void *dWg, void *dWu,
                        void *dWd,
                        int grad_dtype, int accumulate, float *dw, void *workspace,
                        size_t workspace_bytes, void *stream)
{
    const int rc = check_shape(shape);
    if (rc != LORY_OK) return rc;
    if (!X || !w || !Wg || !Wu || !Wd || !dY || !dX || !dWg || !dWu || !dWd || !dw || !workspace)
        return LORY_ERR_NULL;
    if ((G_save == nullptr) != (U_save == nullptr)) return LORY_ERR_NULL;
    if (grad_dtype != LORY_F32 && grad_dtype != LORY_BF16) return LORY_ERR_DTYPE;
    if (shape->dtype == LORY_F32 && grad_dtype != LORY_F32) return LORY_ERR_DTYPE;
    if (accumulate != 0 && accumulate != 1) return LORY_ERR_SHAPE;
    if (!aligned16(X) || !aligned16(w) || !aligned16(Wg) || !aligned16(Wu) || !aligned16(Wd) ||
        !aligned16(dY) || !aligned16(G_save) || !aligned16(U_save) || !aligned16(Wbar_save) ||
        !aligned16(dX) ||
        !aligned16(dWg) || !aligned16(dWu) || !aligned16(dWd) || !aligned16(dw) ||
        !aligned16(workspace))
        return LORY_ERR_ALIGN;
    if (Wbar_save) {
        size_t sb = 0;
        lory_merged_save_bytes(shape, &sb);
        if (sb == 0) return LORY_ERR_SHAPE;
    }
    size_t need = 0;
    lory_workspace_bytes(shape, LORY_PASS_BWD, &need);
    if (workspace_bytes < need) return LORY_ERR_WORKSPACE;
    const Dims m = lory::make_dims(*shape);
    hipStream_t st = (hipStream_t)stream;
    if (m.dtype == LORY_F32)
        return lory::f32_ffn_bwd(m, (const float *)X, w, (const float *)Wg, (const float *)Wu,
                                 (const float *)Wd, (const float *)dY, (const float *)G_save,
                                 (const float *)U_save, (float *)dX, (float *)dWg, (float *)dWu,
                                 (float *)dWd, accumulate, dw, workspace, st);
    return lory::bf16_ffn_bwd(m, X, w, Wg, Wu, Wd, dY, G_save, U_save, Wbar_save, dX, dWg, dWu, dWd,
                              grad_dtype, accumulate, dw, workspace, st);
}

}  // extern "C"
