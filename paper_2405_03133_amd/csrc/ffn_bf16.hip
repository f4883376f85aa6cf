// bf16 merged FFN forward and backward (paper Eq. 1 / Eq. 2, SwiGLU experts):
// host-side orchestration of the MFMA kernels.
//
// Unless the caller asks for them (Wbar_save: the forward then merges straight
// into the caller's buffer and the backward reads them there instead of
// re-merging), the merged parameters of all segments (S * 3 * d * d_ff values)
// are never held at once.  Each pass walks the expert matrices block by block; for a
// block it (1) merges that block for ALL segments into a bounded slab (one read
// of the expert stack, thin MFMA GEMM over the E experts), (2) runs the
// per-segment token GEMMs that consume the slab.  The backward additionally
// produces per-segment weight-gradient slabs that the scatter kernel folds
// into the E expert gradients and into the router-weight gradients at once.
// The slab budget (default 6 GiB) trades workspace for launch size: blocks large enough to
// fill all 256 CUs several times over measured faster than cache-sized blocks.
#include "lory_internal.h"

#include <stdlib.h>

#include "bf16_kernels.h"

namespace lory {

namespace {

using gemm::Params;
using k::EpiGU;
using k::EpiStore;
using k::EpiStore2;
using ms::MergeParams;
using ms::Rect;
using ms::ScatterParams;

typedef uint16_t bf;

size_t g_slab_budget = 0;  // 0 = not initialised yet

size_t slab_budget_bytes()
{
    if (g_slab_budget == 0) {
        size_t mb = 6144;
        if (const char *env = getenv("LORY_SLAB_MB")) {
            const long v = atol(env);
            if (v >= 1 && v <= 16384) mb = (size_t)v;
        }
        g_slab_budget = mb << 20;
    }
    return g_slab_budget;
}

// Which shapes run their token contractions with the merge inside the GEMM (fused_bf16.h) instead
// of the slab pipeline: 0 never, 1 where it measured faster (segments of at most 64 tokens with at
// most 16 experts: the slab pipeline then moves four times the merged parameters of T = 256 through
// HBM for a quarter of the rows each), 2 wherever the shape fits the kernel, 3 like 2 and with the
// backward's per-segment weight gradients kept on chip as well (fsg_kernel; measured slower than the
// slab pipeline at every shape tried, so no other mode uses it).
int g_fused_mode = -1;  // -1 = not initialised yet

int fused_mode()
{
    if (g_fused_mode < 0) {
        int mode = 1;
        if (const char *env = getenv("LORY_FUSED")) {
            const long v = atol(env);
            if (v >= 0 && v <= 3) mode = (int)v;
        }
        g_fused_mode = mode;
    }
    return g_fused_mode;
}

fmg::Params fused_params(const Dims &m, const bf *A0, const bf *A1, int lda, const bf *W0, const bf *W1, int ldw,
                         const float *w, int N, int K, bf *C, int ldc)
{
    fmg::Params p = {};
    p.A[0] = A0; p.A[1] = A1; p.lda[0] = p.lda[1] = lda;
    p.W[0] = W0; p.W[1] = W1;
    p.expert_stride = m.D; p.ldw = ldw;
    p.w = w; p.E = m.E; p.T = m.T; p.tokens = (int)m.tokens;
    p.N = N; p.K = K; p.C = C; p.ldc = ldc;
    return p;
}

bool use_fused(const Dims &m)
{
    const int mode = fused_mode();
    if (mode == 0 || m.tokens > 0x7fffffffL) return false;
    // every contraction of the layer has N and K in {d, d_ff}
    const fmg::Params a = fused_params(m, nullptr, nullptr, m.d, nullptr, nullptr, m.dff, nullptr, m.dff, m.d,
                                       nullptr, m.dff);
    const fmg::Params b = fused_params(m, nullptr, nullptr, m.dff, nullptr, nullptr, m.d, nullptr, m.d, m.dff,
                                       nullptr, m.d);
    if (!k::fused_fits(a) || !k::fused_fits(b)) return false;
    return mode >= 2 || (m.T <= 64 && m.E <= 16);
}

// Whether the backward keeps the per-segment weight gradients on chip as well (fsg_kernel), for
// shapes that kernel takes.
bool use_fused_dw() { return fused_mode() == 3; }

// One fused contraction: C = sum over sources of A_q * Wbar_q(segment), merged on chip.
hipError_t fused_gemm(hipStream_t st, const Dims &m, int cls, const fmg::Params &p, int nsrc, bool w_nc)
{
    const double D = (double)p.N * p.K;
    prof::Range r(st, cls, nsrc * (2.0 * p.tokens * D + 4.0 * m.S * m.E * D),
                  2.0 * (nsrc * ((double)m.E * D + (double)p.tokens * p.K) + (double)p.tokens * p.N));
    return k::launch_fused(st, p, nsrc, w_nc);
}

// Largest multiple of `gran` that is <= limit and <= full, at least gran.
int block_width(size_t budget, size_t bytes_per_unit, int full, int gran)
{
    long wdt = (long)(budget / bytes_per_unit) / gran * gran;
    if (wdt < gran) wdt = gran;
    if (wdt > full) wdt = full;
    return (int)wdt;
}

struct Plan {
    int Sc;        // segments per chunk (limits of the merge / scatter kernels)
    int gran_f;    // granularity of d_ff blocks
    int gran_d;    // granularity of d blocks
    int nf_fwd, jf_fwd, nf_bwd, kf_bwd;
    size_t act;        // bytes of one [chunk tokens, d_ff] bf16 buffer
    size_t slab_fwd;   // bytes of the forward slab region
    size_t slab_bwd;   // bytes of the backward slab region
    size_t partials;   // bytes of the router-weight partial sums
    int prow, pcol;
};

Plan make_plan(const Dims &m)
{
    Plan p;
    const int cap = (m.E <= 32) ? 256 : 128;  // routing-weight operand tables of the merge kernel (LDS)
    p.Sc = m.S < cap ? m.S : cap;
    p.gran_f = (m.dff % 256 == 0) ? 256 : (m.dff % 128 == 0) ? 128 : 64;
    p.gran_d = (m.d % 256 == 0) ? 256 : (m.d % 128 == 0) ? 128 : 64;
    const size_t budget = slab_budget_bytes();
    const size_t S = (size_t)p.Sc;
    p.nf_fwd = block_width(budget, S * m.d * 2 * 2, m.dff, p.gran_f);
    p.jf_fwd = block_width(budget, S * m.dff * 2, m.d, p.gran_d);
    p.nf_bwd = block_width(budget, S * m.d * 2 * 4, m.dff, p.gran_f);
    p.kf_bwd = block_width(budget, S * m.dff * 2 * 2, m.d, p.gran_d);
    p.act = align_up((size_t)p.Sc * m.T * m.dff * 2, 256);
    const size_t gu = S * m.d * p.nf_fwd * 2 * 2, dn = S * m.dff * p.jf_fwd * 2;
    p.slab_fwd = align_up(gu > dn ? gu : dn, 256);
    const size_t ph = S * m.d * p.nf_bwd * 2 * 4, dx = S * m.dff * p.kf_bwd * 2 * 2;
    const size_t re = S * m.d * p.nf_bwd * 2 * 2;  // gate/up slabs when G, U are recomputed
    size_t b = ph > dx ? ph : dx;
    if (re > b) b = re;
    p.slab_bwd = align_up(b, 256);
    k::scatter_partial_dims(p.Sc, m.E, &p.prow, &p.pcol);
    p.partials = align_up((size_t)k::scatter_grid() * p.prow * p.pcol * sizeof(float), 256);
    return p;
}

#define LORY_TRY(expr)                                   \
    do {                                                 \
        if ((expr) != hipSuccess) return LORY_ERR_DEVICE; \
    } while (0)

Rect rect(long D, int pitch, int r0, int nr, int c0, int nc)
{
    Rect rc;
    rc.expert_stride = D;
    rc.pitch = pitch;
    rc.r0 = r0;
    rc.nr = nr;
    rc.c0 = c0;
    rc.nc = nc;
    return rc;
}

double gemm_flops(const Params &p, int nset, int nsrc)
{
    return 2.0 * p.batches * p.M * p.N * p.K * nset * nsrc;
}

hipError_t merge(hipStream_t st, const float *w, int S, int E, const bf *stack, const Rect &rc, bf *slab)
{
    const double n = (double)rc.nr * rc.nc;
    prof::Range r(st, prof::kMerge, 2.0 * S * E * n, 2.0 * n * (E + S));
    MergeParams p;
    p.w = w;
    p.S = S;
    p.E = E;
    p.stack = stack;
    p.rc = rc;
    p.slab = slab;
    p.seg_stride = (long)rc.nr * rc.nc;
    return k::launch_merge(st, p);
}

// Gate/up projections of one d_ff column block for a chunk of segments.
hipError_t gate_up_block(hipStream_t st, const Dims &m, int S, const bf *X, const float *w, const bf *Wg,
                         const bf *Wu, int n0, int nf, bf *slab, bf *G, bf *U, bf *Act, bf *slab_up = nullptr)
{
    bf *sg = slab, *su = slab_up ? slab_up : slab + (size_t)S * m.d * nf;
    const Rect rc = rect(m.D, m.dff, 0, m.d, n0, nf);
    hipError_t e;
    if ((e = merge(st, w, S, m.E, Wg, rc, sg)) != hipSuccess) return e;
    if ((e = merge(st, w, S, m.E, Wu, rc, su)) != hipSuccess) return e;
    Params p = {};
    p.A[0] = X; p.a_batch[0] = (long)m.T * m.d; p.lda[0] = m.d;
    p.B[0] = sg; p.b_batch[0] = (long)m.d * nf; p.ldb[0] = nf;
    p.B[1] = su; p.b_batch[1] = (long)m.d * nf; p.ldb[1] = nf;
    p.M = m.T; p.N = nf; p.K = m.d; p.batches = S;
    // With G and U saved anyway, the activation A = silu(G) * U is cheaper as a streaming pass
    // over them than as a third output plane of the GEMM epilogue; without saved G, U it is
    // computed in the epilogue from the fp32 accumulators.
    const bool split = (G != nullptr && Act != nullptr);
    EpiGU epi = {G, U, split ? nullptr : Act, m.T, m.dff, n0};
    const double out_elems = (double)S * m.T * nf * ((G ? 2 : 0) + ((Act && !split) ? 1 : 0));
    {
        prof::Range r(st, prof::kGemmGU, gemm_flops(p, 2, 1),
                      2.0 * ((double)S * m.T * m.d + 2.0 * S * m.d * nf + out_elems));
        if ((e = k::launch_gu(st, p, epi)) != hipSuccess) return e;
    }
    if (split) {
        prof::Range r(st, prof::kSwigluFwd, 4.0 * S * m.T * nf, 2.0 * 3.0 * S * m.T * nf);
        return k::launch_swiglu_fwd(st, G, U, Act, (long)S * m.T, m.dff, n0, nf);
    }
    return hipSuccess;
}

}  // namespace

int set_fused_mode(int mode)
{
    if (mode < 0 || mode > 3) return LORY_ERR_SHAPE;
    g_fused_mode = mode;
    return LORY_OK;
}

int set_slab_budget(size_t bytes)
{
    if (bytes < ((size_t)64 << 10)) return LORY_ERR_SHAPE;
    g_slab_budget = bytes;
    return LORY_OK;
}

size_t bf16_merged_save_bytes(const Dims &m)
{
    const Plan p = make_plan(m);
    if (m.S > p.Sc) return 0;  // more segments than one merge launch handles
    return (size_t)3 * m.S * m.D * 2;
}

size_t bf16_workspace_bytes(const Dims &m, int pass)
{
    const Plan p = make_plan(m);
    if (pass == LORY_PASS_FWD) {
        // fused path: G and U of all tokens when the caller does not keep them
        const size_t gu = use_fused(m) ? 2 * p.act : 0;
        return p.act + (p.slab_fwd > gu ? p.slab_fwd : gu);
    }
    // dG, dU, Act, recomputed G and U, slabs, router-weight partial sums
    return 5 * p.act + p.slab_bwd + p.partials;
}

int bf16_ffn_fwd(const Dims &m, const void *Xv, const float *w, const void *Wgv, const void *Wuv,
                 const void *Wdv, void *Yv, void *Gv, void *Uv, void *Wbarv, void *ws, hipStream_t st)
{
    Plan pl = make_plan(m);
    bf *Wbar = (bf *)Wbarv;  // [Wg_bar | Wu_bar | Wd_bar], each [S][rows][cols]; doubles as the slab
    if (Wbar) {
        pl.nf_fwd = m.dff;
        pl.jf_fwd = m.d;
    }
    const bf *X = (const bf *)Xv, *Wg = (const bf *)Wgv, *Wu = (const bf *)Wuv, *Wd = (const bf *)Wdv;
    bf *Y = (bf *)Yv, *G = (bf *)Gv, *U = (bf *)Uv;
    bf *Act = (bf *)ws;
    bf *slab = (bf *)((char *)ws + pl.act);
    const long TD = (long)m.T * m.d, TF = (long)m.T * m.dff;

    if (!Wbar && m.S <= pl.Sc && use_fused(m)) {
        // merged parameters never leave the chip: three fused contractions and one SwiGLU pass
        bf *Gf = G ? G : slab, *Uf = U ? U : (bf *)((char *)slab + pl.act);
        LORY_TRY(fused_gemm(st, m, prof::kFusedGU,
                            fused_params(m, X, nullptr, m.d, Wg, nullptr, m.dff, w, m.dff, m.d, Gf, m.dff), 1, true));
        LORY_TRY(fused_gemm(st, m, prof::kFusedGU,
                            fused_params(m, X, nullptr, m.d, Wu, nullptr, m.dff, w, m.dff, m.d, Uf, m.dff), 1, true));
        {
            prof::Range r(st, prof::kSwigluFwd, 4.0 * m.tokens * m.dff, 2.0 * 3.0 * m.tokens * m.dff);
            LORY_TRY(k::launch_swiglu_fwd(st, Gf, Uf, Act, m.tokens, m.dff, 0, m.dff));
        }
        LORY_TRY(fused_gemm(st, m, prof::kFusedDown,
                            fused_params(m, Act, nullptr, m.dff, Wd, nullptr, m.d, w, m.d, m.dff, Y, m.d), 1, true));
        return LORY_OK;
    }

    for (int s0 = 0; s0 < m.S; s0 += pl.Sc) {
        const int S = (m.S - s0 < pl.Sc) ? (m.S - s0) : pl.Sc;
        const float *wc = w + (size_t)s0 * m.E;
        const bf *Xc = X + (size_t)s0 * TD;
        bf *Gc = G ? G + (size_t)s0 * TF : nullptr;
        bf *Uc = U ? U + (size_t)s0 * TF : nullptr;
        // gate / up projections + SwiGLU, one d_ff column block at a time
        for (int n0 = 0; n0 < m.dff; n0 += pl.nf_fwd) {
            const int nf = (m.dff - n0 < pl.nf_fwd) ? (m.dff - n0) : pl.nf_fwd;
            if (Wbar)
                LORY_TRY(gate_up_block(st, m, S, Xc, wc, Wg, Wu, n0, nf, Wbar, Gc, Uc, Act,
                                       Wbar + (size_t)m.S * m.D));
            else
                LORY_TRY(gate_up_block(st, m, S, Xc, wc, Wg, Wu, n0, nf, slab, Gc, Uc, Act));
        }
        // down projection, one block of output columns at a time
        for (int j0 = 0; j0 < m.d; j0 += pl.jf_fwd) {
            const int jf = (m.d - j0 < pl.jf_fwd) ? (m.d - j0) : pl.jf_fwd;
            bf *sd = Wbar ? Wbar + (size_t)2 * m.S * m.D : slab;
            LORY_TRY(merge(st, wc, S, m.E, Wd, rect(m.D, m.d, 0, m.dff, j0, jf), sd));
            Params p = {};
            p.A[0] = Act; p.a_batch[0] = TF; p.lda[0] = m.dff;
            p.B[0] = sd; p.b_batch[0] = (long)m.dff * jf; p.ldb[0] = jf;
            p.M = m.T; p.N = jf; p.K = m.dff; p.batches = S;
            EpiStore epi = {Y + (size_t)s0 * TD + j0, TD, m.d};
            prof::Range r(st, prof::kGemmDown, gemm_flops(p, 1, 1),
                          2.0 * ((double)S * TF + (double)S * m.dff * jf + (double)S * m.T * jf));
            LORY_TRY(k::launch_down(st, p, epi));
        }
    }
    return LORY_OK;
}

// Merged parameters of all m.S segments, materialised as [Wg_bar | Wu_bar | Wd_bar], each
// [S][rows][cols] (the layout of Wbar_save).
int bf16_merge_all(const Dims &m, const float *w, const void *Wgv, const void *Wuv, const void *Wdv,
                   void *Wbarv, hipStream_t st)
{
    const Plan pl = make_plan(m);
    const bf *stacks[3] = {(const bf *)Wgv, (const bf *)Wuv, (const bf *)Wdv};
    const Rect rcs[3] = {rect(m.D, m.dff, 0, m.d, 0, m.dff), rect(m.D, m.dff, 0, m.d, 0, m.dff),
                         rect(m.D, m.d, 0, m.dff, 0, m.d)};
    bf *out = (bf *)Wbarv;
    for (int s0 = 0; s0 < m.S; s0 += pl.Sc) {
        const int S = (m.S - s0 < pl.Sc) ? (m.S - s0) : pl.Sc;
        for (int x = 0; x < 3; ++x)
            LORY_TRY(merge(st, w + (size_t)s0 * m.E, S, m.E, stacks[x], rcs[x],
                           out + ((size_t)x * m.S + s0) * m.D));
    }
    return LORY_OK;
}

size_t bf16_dense_workspace_bytes(const Dims &m) { return align_up((size_t)m.tokens * m.dff * 2, 256); }

// Dense SwiGLU FFN of every sequence with its own materialised merged parameters
// (m.T == m.L: one parameter set per sequence, T a multiple of 64).
int bf16_dense_ffn_fwd(const Dims &m, const void *Xv, const void *Wbarv, void *Yv, void *ws, hipStream_t st)
{
    const bf *X = (const bf *)Xv, *Wbar = (const bf *)Wbarv;
    bf *Y = (bf *)Yv, *Act = (bf *)ws;
    const long TD = (long)m.T * m.d, TF = (long)m.T * m.dff;
    {
        Params p = {};
        p.A[0] = X; p.a_batch[0] = TD; p.lda[0] = m.d;
        p.B[0] = Wbar; p.b_batch[0] = m.D; p.ldb[0] = m.dff;
        p.B[1] = Wbar + (size_t)m.S * m.D; p.b_batch[1] = m.D; p.ldb[1] = m.dff;
        p.M = m.T; p.N = m.dff; p.K = m.d; p.batches = m.S;
        EpiGU epi = {nullptr, nullptr, Act, m.T, m.dff, 0};
        prof::Range r(st, prof::kGemmGU, gemm_flops(p, 2, 1),
                      2.0 * ((double)m.S * TD + 2.0 * m.S * m.D + (double)m.S * TF));
        LORY_TRY(k::launch_gu(st, p, epi));
    }
    {
        Params p = {};
        p.A[0] = Act; p.a_batch[0] = TF; p.lda[0] = m.dff;
        p.B[0] = Wbar + (size_t)2 * m.S * m.D; p.b_batch[0] = m.D; p.ldb[0] = m.d;
        p.M = m.T; p.N = m.d; p.K = m.dff; p.batches = m.S;
        EpiStore epi = {Y, TD, m.d};
        prof::Range r(st, prof::kGemmDown, gemm_flops(p, 1, 1),
                      2.0 * ((double)m.S * TF + (double)m.S * m.D + (double)m.S * TD));
        LORY_TRY(k::launch_down(st, p, epi));
    }
    return LORY_OK;
}

int bf16_ffn_bwd(const Dims &m, const void *Xv, const float *w, const void *Wgv, const void *Wuv,
                 const void *Wdv, const void *dYv, const void *Gv, const void *Uv, const void *Wbarv,
                 void *dXv, void *dWg, void *dWu, void *dWd, int grad_dtype, int accumulate, float *dw,
                 void *ws, hipStream_t st)
{
    // saved merged parameters [Wg_bar | Wu_bar | Wd_bar]: no re-merge, the GEMMs read them in place
    const bf *Wbar = (const bf *)Wbarv;
    const bf *Wbar_g = Wbar, *Wbar_u = Wbar ? Wbar + (size_t)m.S * m.D : nullptr;
    const bf *Wbar_d = Wbar ? Wbar + (size_t)2 * m.S * m.D : nullptr;
    const Plan pl = make_plan(m);
    const bf *X = (const bf *)Xv, *Wg = (const bf *)Wgv, *Wu = (const bf *)Wuv, *Wd = (const bf *)Wdv;
    const bf *dY = (const bf *)dYv, *G = (const bf *)Gv, *U = (const bf *)Uv;
    bf *dX = (bf *)dXv;
    char *base = (char *)ws;
    bf *dG = (bf *)base, *dU = (bf *)(base + pl.act), *Act = (bf *)(base + 2 * pl.act);
    bf *Gr = (bf *)(base + 3 * pl.act), *Ur = (bf *)(base + 4 * pl.act);
    bf *slab = (bf *)(base + 5 * pl.act);
    float *partials = (float *)(base + 5 * pl.act + pl.slab_bwd);
    const long TD = (long)m.T * m.d, TF = (long)m.T * m.dff;
    const int grid = k::scatter_grid();
    const int grad_f32 = (grad_dtype == LORY_F32) ? 1 : 0;
    // token contractions with the merge inside the GEMM (no re-merged slabs); the per-segment weight
    // gradients still pass through the slab
    const bool fused = !Wbar && m.S <= pl.Sc && use_fused(m);
    // ... unless the expert-gradient kernel that keeps them on chip takes the shape (bf16 gradients
    // that overwrite; at most 16 experts)
    auto dw_params = [&](const bf *A, int lda, const bf *B, int ldb, const bf *W, void *dW, int M, int N) {
        fsg::Params q = {};
        q.A = (const uint16_t *)A; q.lda = lda;
        q.B = (const uint16_t *)B; q.ldb = ldb;
        q.W = (const uint16_t *)W; q.dW = (uint16_t *)dW;
        q.expert_stride = (long)m.D; q.ldw = N;
        q.w = w; q.E = m.E; q.T = m.T; q.S = m.S; q.M = M; q.N = N;
        return q;
    };
    const bool fused_dw = fused && use_fused_dw() && !grad_f32 && !accumulate &&
                          k::fused_dw_fits(dw_params(nullptr, m.dff, nullptr, m.d, nullptr, nullptr, m.dff, m.d)) &&
                          k::fused_dw_fits(dw_params(nullptr, m.d, nullptr, m.dff, nullptr, nullptr, m.d, m.dff));

    for (int s0 = 0; s0 < m.S; s0 += pl.Sc) {
        const int S = (m.S - s0 < pl.Sc) ? (m.S - s0) : pl.Sc;
        const float *wc = w + (size_t)s0 * m.E;
        const bf *Xc = X + (size_t)s0 * TD;
        const bf *dYc = dY + (size_t)s0 * TD;
        const int acc_dW = (accumulate || s0 > 0) ? 1 : 0;
        int partials_add = 0;

        const bf *Gc, *Uc;
        if (G && U) {
            Gc = G + (size_t)s0 * TF;
            Uc = U + (size_t)s0 * TF;
        } else if (fused) {
            LORY_TRY(fused_gemm(st, m, prof::kFusedGU,
                                fused_params(m, X, nullptr, m.d, Wg, nullptr, m.dff, w, m.dff, m.d, Gr, m.dff), 1, true));
            LORY_TRY(fused_gemm(st, m, prof::kFusedGU,
                                fused_params(m, X, nullptr, m.d, Wu, nullptr, m.dff, w, m.dff, m.d, Ur, m.dff), 1, true));
            Gc = Gr;
            Uc = Ur;
        } else {
            // the backward slab region holds four slabs of nf_bwd columns, i.e. a gate and an
            // up slab of 2 * nf_bwd columns each
            const int step = 2 * pl.nf_bwd;
            for (int n0 = 0; n0 < m.dff; n0 += step) {
                const int nf = (m.dff - n0 < step) ? (m.dff - n0) : step;
                LORY_TRY(gate_up_block(st, m, S, Xc, wc, Wg, Wu, n0, nf, slab, Gr, Ur, nullptr));
            }
            Gc = Gr;
            Uc = Ur;
        }

        if (fused) {
            // dA = dY Wd_bar^T for all of d_ff at once (Wd[e] is [d_ff][d]: K contiguous), then the
            // SwiGLU backward pass: dG, dU, A
            LORY_TRY(fused_gemm(st, m, prof::kFusedDA,
                                fused_params(m, dY, nullptr, m.d, Wd, nullptr, m.d, w, m.dff, m.d, dG, m.dff), 1, false));
            prof::Range r2(st, prof::kSwigluBwd, 12.0 * m.tokens * m.dff, 2.0 * 6.0 * m.tokens * m.dff);
            LORY_TRY(k::launch_swiglu_bwd(st, Gc, Uc, dG, dU, Act, m.tokens, m.dff, 0, m.dff));
        }

        if (fused_dw) {
            // expert gradients and routing-weight inner products of the three matrices, the per-segment
            // weight gradients never leaving the CU; every workgroup-wave adds its inner products
            // to a slot of its own, matrix after matrix
            fsg::Params q[3] = {dw_params(Act, m.dff, dY, m.d, Wd, dWd, m.dff, m.d),
                                dw_params(X, m.d, dG, m.dff, Wg, dWg, m.d, m.dff),
                                dw_params(X, m.d, dU, m.dff, Wu, dWu, m.d, m.dff)};
            int slots = 0;
            for (int i = 0; i < 3; ++i) {
                q[i].partials = partials;
                q[i].partials_add = i > 0;
                slots = k::fused_dw_slots(q[i]);   // the same for the three matrices (M N is)
                const double n = (double)m.D;
                prof::Range r(st, prof::kFusedDW, 2.0 * m.tokens * n + 8.0 * m.S * 16 * n,
                              2.0 * (2.0 * m.E * n + (double)m.tokens * (m.d + m.dff)));
                LORY_TRY(k::launch_fused_dw(st, q[i]));
            }
            prof::Range r(st, prof::kDwReduce, (double)slots * m.S * m.E, 4.0 * slots * m.S * 16);
            LORY_TRY(k::launch_dw_reduce(st, partials, slots, m.S, 16, dw, m.S, m.E));
        }

        // ---- d_ff blocks: dA (+ SwiGLU backward), weight-gradient slabs, scatter
        for (int n0 = 0; !fused_dw && n0 < m.dff; n0 += pl.nf_bwd) {
            const int nf = (m.dff - n0 < pl.nf_bwd) ? (m.dff - n0) : pl.nf_bwd;
            const size_t blk = (size_t)S * m.d * nf;  // elements of one slab of this block
            bf *s_md = slab, *s_gd = slab + blk, *s_gg = slab + 2 * blk, *s_gu = slab + 3 * blk;
            const Rect rows_d = rect(m.D, m.d, n0, nf, 0, m.d);      // rows n0.. of Wd [d_ff, d]
            const Rect cols_f = rect(m.D, m.dff, 0, m.d, n0, nf);    // columns n0.. of Wg/Wu [d, d_ff]

            // dA = dY Wd_bar^T for these d_ff columns, then the SwiGLU backward pass: dG, dU, A
            if (!Wbar && !fused) LORY_TRY(merge(st, wc, S, m.E, Wd, rows_d, s_md));
            if (!fused) {
                Params p = {};
                p.A[0] = dYc; p.a_batch[0] = TD; p.lda[0] = m.d;
                p.B[0] = Wbar ? Wbar_d + (size_t)n0 * m.d : s_md;
                p.b_batch[0] = Wbar ? m.D : (long)nf * m.d;
                p.ldb[0] = m.d;
                p.M = m.T; p.N = nf; p.K = m.d; p.batches = S;
                EpiStore epi = {dG + n0, TF, m.dff};  // dA parks in the dG buffer
                {
                    prof::Range r(st, prof::kGemmDA, gemm_flops(p, 1, 1),
                                  2.0 * ((double)S * TD + (double)S * nf * m.d + (double)S * m.T * nf));
                    LORY_TRY(k::launch_da(st, p, epi));
                }
                prof::Range r2(st, prof::kSwigluBwd, 12.0 * S * m.T * nf, 2.0 * 6.0 * S * m.T * nf);
                LORY_TRY(k::launch_swiglu_bwd(st, Gc, Uc, dG, dU, Act, (long)S * m.T, m.dff, n0, nf));
            }
            // dWd_bar rows = A^T dY
            {
                Params p = {};
                p.A[0] = Act + n0; p.a_batch[0] = TF; p.lda[0] = m.dff;
                p.B[0] = dYc; p.b_batch[0] = TD; p.ldb[0] = m.d;
                p.M = nf; p.N = m.d; p.K = m.T; p.batches = S;
                EpiStore epi = {s_gd, (long)nf * m.d, m.d};
                prof::Range r(st, prof::kGemmDWD, gemm_flops(p, 1, 1),
                              2.0 * ((double)S * m.T * nf + (double)S * TD + (double)S * nf * m.d));
                LORY_TRY(k::launch_dwd(st, p, epi));
            }
            // dWg_bar, dWu_bar columns = X^T dG, X^T dU
            {
                Params p = {};
                p.A[0] = Xc; p.a_batch[0] = TD; p.lda[0] = m.d;
                p.B[0] = dG + n0; p.b_batch[0] = TF; p.ldb[0] = m.dff;
                p.B[1] = dU + n0; p.b_batch[1] = TF; p.ldb[1] = m.dff;
                p.M = m.d; p.N = nf; p.K = m.T; p.batches = S;
                EpiStore2 epi = {s_gg, s_gu, (long)m.d * nf, nf};
                prof::Range r(st, prof::kGemmDWGU, gemm_flops(p, 2, 1),
                              2.0 * ((double)S * TD + 2.0 * S * m.T * nf + 2.0 * S * m.d * nf));
                LORY_TRY(k::launch_dwgu(st, p, epi));
            }
            // E-way scatter and router-weight inner products
            const bf *stacks[3] = {Wd, Wg, Wu};
            void *grads[3] = {dWd, dWg, dWu};
            const bf *gsl[3] = {s_gd, s_gg, s_gu};
            const Rect rcs[3] = {rows_d, cols_f, cols_f};
            for (int i = 0; i < 3; ++i) {
                const int padd = partials_add;
                for (int e0 = 0; e0 < m.E; e0 += 32) {  // windows of 32 experts
                    ScatterParams sp;
                    sp.w = wc; sp.S = S; sp.E = m.E; sp.e0 = e0;
                    sp.gslab = gsl[i]; sp.seg_stride = (long)rcs[i].nr * rcs[i].nc;
                    sp.stack = stacks[i]; sp.dW = grads[i]; sp.rc = rcs[i];
                    sp.grad_f32 = grad_f32; sp.accumulate = acc_dW;
                    sp.partials = partials; sp.pcols = pl.pcol; sp.partials_add = padd;
                    const int win = (m.E - e0 < 32) ? (m.E - e0) : 32;
                    const double n = (double)rcs[i].nr * rcs[i].nc;
                    const double gsz = grad_f32 ? 4.0 : 2.0;
                    prof::Range r(st, prof::kScatter, 4.0 * S * win * n,
                                  2.0 * n * (S + win) + gsz * n * win * (acc_dW ? 2 : 1));
                    LORY_TRY(k::launch_scatter(st, sp, grid));
                }
                partials_add = 1;
            }
        }

        if (fused) {
            // dX = dG Wg_bar^T + dU Wu_bar^T: two sources, Wg[e] / Wu[e] are [d][d_ff] (K contiguous)
            LORY_TRY(fused_gemm(st, m, prof::kFusedDX,
                                fused_params(m, dG, dU, m.dff, Wg, Wu, m.dff, w, m.d, m.dff, dX, m.d), 2, false));
        }
        // ---- dX = dG Wg_bar^T + dU Wu_bar^T, one block of d columns at a time
        for (int k0 = 0; !fused && k0 < m.d; k0 += pl.kf_bwd) {
            const int kf = (m.d - k0 < pl.kf_bwd) ? (m.d - k0) : pl.kf_bwd;
            const size_t blk = (size_t)S * kf * m.dff;
            bf *s_g = slab, *s_u = slab + blk;
            const Rect rows = rect(m.D, m.dff, k0, kf, 0, m.dff);
            if (!Wbar) {
                LORY_TRY(merge(st, wc, S, m.E, Wg, rows, s_g));
                LORY_TRY(merge(st, wc, S, m.E, Wu, rows, s_u));
            }
            Params p = {};
            p.A[0] = dG; p.a_batch[0] = TF; p.lda[0] = m.dff;
            p.A[1] = dU; p.a_batch[1] = TF; p.lda[1] = m.dff;
            p.B[0] = Wbar ? Wbar_g + (size_t)k0 * m.dff : s_g;
            p.B[1] = Wbar ? Wbar_u + (size_t)k0 * m.dff : s_u;
            p.b_batch[0] = p.b_batch[1] = Wbar ? m.D : (long)kf * m.dff;
            p.ldb[0] = p.ldb[1] = m.dff;
            p.M = m.T; p.N = kf; p.K = m.dff; p.batches = S;
            EpiStore epi = {dX + (size_t)s0 * TD + k0, TD, m.d};
            prof::Range r(st, prof::kGemmDX, gemm_flops(p, 1, 2),
                          2.0 * (2.0 * S * TF + 2.0 * S * kf * m.dff + (double)S * m.T * kf));
            LORY_TRY(k::launch_dx(st, p, epi));
        }

        if (!fused_dw) {
            int prow, pcol;
            k::scatter_partial_dims(S, m.E, &prow, &pcol);
            prof::Range r(st, prof::kDwReduce, (double)grid * S * m.E, 4.0 * grid * prow * pcol);
            LORY_TRY(k::launch_dw_reduce(st, partials, grid, prow, pcol, dw + (size_t)s0 * m.E, S, m.E));
        }
    }
    return LORY_OK;
}

}  // namespace lory
