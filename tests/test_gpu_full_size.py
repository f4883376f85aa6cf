"""Parity at the benchmark's full sizes, in the launch configurations bench.py
times (default slab budget; saved G/U; merged parameters re-merged by the
backward, or saved for it), checked on sampled outputs that the fp64 oracle
can compute one by one:

  * routing weights: all of them (the oracle's route is cheap);
  * Y, dX, dw, G, U of sampled segments: a segment is a layer of its own
    (B = 1, L = T) once its routing-weight row is given;
  * dWg[:, :, J], dWu[:, :, J], dWd[:, J, :], G[:, J], U[:, J] for sampled
    blocks J of d_ff columns: restricting the experts to J is again a Lory
    layer (d_ff' = |J|) whose weight gradients, for the same dY, are the full
    layer's restricted to J;
  * for EVERY segment, an identity between outputs that needs no oracle:
        sum_e w[s,e] dw[s,e] = <Y_s, dY_s> + <X_s, dX_s>
    (<Wd_bar, dWd_bar> = <Y, dY>; <Wu_bar, dWu_bar> = <U, dU> = <A, dA> = <Y, dY>;
    <Wg_bar, dWg_bar> = <G, dG>; and <X, dX> = <G, dG> + <U, dU>).

Every sampled tensor passes parity_util.check: whole-tensor rel-L2, worst-row
rel-L2 and largest absolute error.
"""
import numpy as np
import pytest
import torch

from oracle import lory_oracle as orc
from paper_2405_03133_amd import binding as lb
from paper_2405_03133_amd.inputs import CONFIGS, make_inputs
from parity_util import check, host, rel_l2

pytestmark = pytest.mark.gpu
TOL = 1e-2
# Identity bar.  Each side is a sum of n products of nearly independent factors, so its size is
# about ||a|| ||b|| / sqrt(n) of the factors, and an error of relative size eps in one factor moves
# it by eps times that.  With eps = 4e-3 observed for the bf16 tensors, three such terms and a
# margin of about six standard deviations over the segments of a run: 3e-2 of the summed term
# sizes.  (A left side of zero misses the bar by a factor of thirty.)
ID_TOL = 3e-2

# (configuration, mode, structured inputs); modes: "remerge" = bench.py's default launch
# configuration (G/U saved, the backward re-merges; short segments take the merge-inside-the-GEMM
# kernels by the library's own rule), "saved" = merged parameters handed to the backward (bench.py
# --merged-save), "fwd" = route + forward with nothing saved, "fused" = as "remerge" with the
# merge-inside-the-GEMM kernels forced on (bench.py --fused 2), "fused_all" = with the expert-gradient
# kernel that keeps the per-segment weight gradients on chip as well (bench.py --fused 3).
CASES = [
    ("C4", "remerge", False),
    ("C4", "fused", False),
    ("C5_T128", "fused", True),
    ("C5_T64", "fused_all", False),
    ("C4", "saved", True),
    ("C2", "fwd", False),
    ("C3", "remerge", True),
    ("C4_EP8", "remerge", False),
    ("C5_T64", "remerge", False),
    ("C5_T128", "remerge", False),
    ("C5_T256", "remerge", True),
    ("C5_T512", "remerge", False),
    ("C5_T1024", "saved", False),
    ("P15_E8", "saved", False),
    ("P15_E16", "remerge", False),
    ("P15_E32", "remerge", True),
    ("P7_E4", "remerge", False),
    ("C4_T64", "remerge", False),
]


def term_size(a, b):
    """Size of <a_s, b_s> per segment for nearly independent factors: ||a_s|| ||b_s|| / sqrt(n)."""
    n = a.shape[1]
    return np.linalg.norm(a, axis=1) * np.linalg.norm(b, axis=1) / np.sqrt(n)


@pytest.mark.timeout(1500)
@pytest.mark.parametrize("name,mode,structured", CASES, ids=[f"{c[0]}-{c[1]}{'-structured' if c[2] else ''}" for c in CASES])
def test_full_size_sampled(name, mode, structured):
    cfg = CONFIGS[name]
    print(f"[full] generating {cfg} mode={mode} structured={structured}", flush=True)
    t = make_inputs(cfg, structured=structured, with_dy=(mode != "fwd"))
    dev = {k: torch.from_numpy(v).cuda().to(torch.bfloat16).contiguous() for k, v in t.items()}
    shape = lb.make_shape(cfg.B, cfg.L, cfg.T, cfg.d, cfg.d_ff, cfg.E, torch.bfloat16)
    print("[full] running GPU route/fwd/bwd", flush=True)
    lb.lory_set_fused_merge({"fused": 2, "fused_all": 3}.get(mode, 1))
    try:
        results = _run_gpu(cfg, dev, shape, mode)
    finally:
        lb.lory_set_fused_merge(1)
    w, Y, G, U, dX, dWg, dWu, dWd, dw = results
    _compare(name, cfg, t, mode, w, Y, G, U, dX, dWg, dWu, dWd, dw)


def _run_gpu(cfg, dev, shape, mode):
    w = lb.lory_route(dev["X"], dev["R"], cfg.T, d_ff=cfg.d_ff)
    G = U = Wbar = None
    if mode != "fwd":
        G = torch.empty((cfg.tokens, cfg.d_ff), dtype=torch.bfloat16, device="cuda")
        U = torch.empty_like(G)
    if mode == "saved":
        Wbar = lb.alloc_merged_save(shape)
        assert Wbar is not None
    Y = lb.lory_merged_ffn_fwd(dev["X"], w, dev["Wg"], dev["Wu"], dev["Wd"], cfg.T, G_save=G, U_save=U,
                               Wbar_save=Wbar)
    dX = dWg = dWu = dWd = dw = None
    if mode != "fwd":
        dX, dWg, dWu, dWd, dw = lb.lory_merged_ffn_bwd(dev["X"], w, dev["Wg"], dev["Wu"], dev["Wd"], dev["dY"],
                                                       cfg.T, G_save=G, U_save=U, grad_dtype=torch.bfloat16,
                                                       Wbar_save=Wbar)
    torch.cuda.synchronize()
    return w, Y, G, U, dX, dWg, dWu, dWd, dw


def _compare(name, cfg, t, mode, w, Y, G, U, dX, dWg, dWu, dWd, dw):
    w_h = host(w)

    # ---- routing weights, all of them
    ref_w = orc.route(t["X"], t["R"], cfg.T)["w"]
    check(f"{name} w", w_h, ref_w, 1e-5)
    np.testing.assert_allclose(w_h.sum(-1), 1.0, atol=1e-5)
    print(f"[full] mean of the largest routing weight {w_h.max(-1).mean():.3f} (1/E = {1.0 / cfg.E:.3f})", flush=True)

    Xs = t["X"].reshape(cfg.S, cfg.T, cfg.d)
    seg = lambda a, width: a.reshape(cfg.S, cfg.T, width)
    segments = sorted({min(5, cfg.S - 1), cfg.S - 1})

    if mode == "fwd":
        for s in segments:
            print(f"[full] oracle on segment {s}", flush=True)
            f = orc.ffn_fwd(Xs[s], w_h[s:s + 1], t["Wg"], t["Wu"], t["Wd"], cfg.T)
            check(f"{name} segment {s} Y", host(seg(Y, cfg.d)[s]), f["Y"], TOL)
        # a block of d_ff columns is a layer of its own whose output is one term of Y; its G and U
        # are not returned in this mode, so the forward is sampled by segments only
        return

    # ---- identity between outputs, every segment
    dw_h = host(dw)
    Yh, dYh = host(Y).reshape(cfg.S, -1), t["dY"].astype(np.float64).reshape(cfg.S, -1)
    Xh, dXh = t["X"].astype(np.float64).reshape(cfg.S, -1), host(dX).reshape(cfg.S, -1)
    lhs = (w_h * dw_h).sum(-1)
    rhs = (Yh * dYh).sum(-1) + (Xh * dXh).sum(-1)
    size = (term_size(Yh, dYh) + term_size(Xh, dXh)
            + np.linalg.norm(w_h, axis=1) * np.linalg.norm(dw_h, axis=1))
    worst = float(np.max(np.abs(lhs - rhs) / size))
    print(f"[full] identity sum_e w dw = <Y,dY> + <X,dX>: worst |difference| / term size {worst:.2e} "
          f"over {cfg.S} segments (a zero left side would read {float(np.max(np.abs(rhs) / size)):.2f})",
          flush=True)
    assert worst <= ID_TOL, worst
    del Yh, dYh, Xh, dXh

    # ---- sampled segments: Y, dX, dw, G, U
    dYs = t["dY"].reshape(cfg.S, cfg.T, cfg.d)
    for s in segments:
        print(f"[full] oracle on segment {s}", flush=True)
        f = orc.ffn_fwd(Xs[s], w_h[s:s + 1], t["Wg"], t["Wu"], t["Wd"], cfg.T, want_gu=True)
        g = orc.ffn_bwd(Xs[s], w_h[s:s + 1], t["Wg"], t["Wu"], t["Wd"], dYs[s], cfg.T)
        check(f"{name} segment {s} Y", host(seg(Y, cfg.d)[s]), f["Y"], TOL)
        check(f"{name} segment {s} dX", host(seg(dX, cfg.d)[s]), g["dX"], TOL)
        check(f"{name} segment {s} dw", dw_h[s], g["dw"][0], TOL)
        check(f"{name} segment {s} G", host(seg(G, cfg.d_ff)[s]), f["G"], TOL)
        check(f"{name} segment {s} U", host(seg(U, cfg.d_ff)[s]), f["U"], TOL)
        del f, g

    # ---- sampled d_ff blocks: weight gradients (all experts, all rows) and saved activations
    for j0 in sorted({0, cfg.d_ff - 192}):
        J = slice(j0, j0 + 64)
        print(f"[full] oracle on d_ff block {j0}..{j0 + 64}", flush=True)
        Wg_j = np.ascontiguousarray(t["Wg"][:, :, J])
        Wu_j = np.ascontiguousarray(t["Wu"][:, :, J])
        Wd_j = np.ascontiguousarray(t["Wd"][:, J, :])
        f = orc.ffn_fwd(t["X"], w_h, Wg_j, Wu_j, Wd_j, cfg.T, want_gu=True)
        g = orc.ffn_bwd(t["X"], w_h, Wg_j, Wu_j, Wd_j, t["dY"], cfg.T)
        check(f"{name} block {j0} dWg", host(dWg[:, :, J]), g["dWg"], TOL)
        check(f"{name} block {j0} dWu", host(dWu[:, :, J]), g["dWu"], TOL)
        check(f"{name} block {j0} dWd", host(dWd[:, J, :]), g["dWd"], TOL)
        check(f"{name} block {j0} G", host(G[:, J]), f["G"], TOL)
        check(f"{name} block {j0} U", host(U[:, J]), f["U"], TOL)
        del f, g
