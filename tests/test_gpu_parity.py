"""GPU parity: the HIP library (through the C ABI) against the CPU fp64
oracle, element by element on the same seeded inputs.

Tolerances (relative L2 per output tensor): 1e-5 for the fp32 configuration,
1e-2 for bf16 operands with fp32 accumulation.
"""
import numpy as np
import pytest
import torch

from oracle import lory_oracle as orc
from paper_2405_03133_amd import binding as lb
from paper_2405_03133_amd.inputs import CONFIGS, LoryConfig, make_inputs, make_routing_weights, round_to_bf16
from parity_util import check, host, rel_l2

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 1e-2}
# Router-weight gradient of the whole layer: dR = sum_s hbar_s^T dz_s, dz = e * (de - <e, de>), de = the
# FFN's dw shifted by one segment.  It inherits the error of dw (the bar above; the centring
# de - <e, de> is well conditioned for these inputs, ||de|| / ||de - <e, de>|| is about 1) and of the
# fp32 softmax and segment means of the forward (1e-7 relative), hence 1e-4 instead of 1e-5 for the
# fp32 configuration, as for lory_route_bwd on its own.
DR_TOL = {"f32": 1e-4, "bf16": 1e-2}


def tdtype(cfg):
    return torch.float32 if cfg.dtype == "f32" else torch.bfloat16


def to_dev(a, cfg):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda().to(tdtype(cfg)).contiguous()


def run_layer(cfg, t, w_override=None, save=True, grad_dtype=torch.float32, merged_save=False):
    """route -> fwd -> bwd on the GPU through the C ABI; returns numpy float64."""
    print(f"[gpu] {cfg}", flush=True)
    X, R = to_dev(t["X"], cfg), to_dev(t["R"], cfg)
    Wg, Wu, Wd = (to_dev(t[k], cfg) for k in ("Wg", "Wu", "Wd"))
    dY = to_dev(t["dY"], cfg)
    hbar = torch.empty((cfg.S, cfg.d), dtype=torch.float32, device="cuda")
    w = lb.lory_route(X, R, cfg.T, hbar=hbar, d_ff=cfg.d_ff)
    w_used = w if w_override is None else torch.from_numpy(w_override).cuda().float().contiguous()
    G = U = None
    if save:
        G = torch.empty((cfg.tokens, cfg.d_ff), dtype=X.dtype, device="cuda")
        U = torch.empty_like(G)
    Wbar = None
    if merged_save:
        Wbar = lb.alloc_merged_save(lb.make_shape(cfg.B, cfg.L, cfg.T, cfg.d, cfg.d_ff, cfg.E, X.dtype))
        assert Wbar is not None
    Y = lb.lory_merged_ffn_fwd(X, w_used, Wg, Wu, Wd, cfg.T, G_save=G, U_save=U, Wbar_save=Wbar)
    dX, dWg, dWu, dWd, dw = lb.lory_merged_ffn_bwd(X, w_used, Wg, Wu, Wd, dY, cfg.T, G_save=G, U_save=U,
                                                   grad_dtype=grad_dtype, Wbar_save=Wbar)
    torch.cuda.synchronize()
    out = {"w": host(w), "hbar": host(hbar), "Y": host(Y), "dX": host(dX), "dWg": host(dWg),
           "dWu": host(dWu), "dWd": host(dWd), "dw": host(dw), "w_used": host(w_used)}
    if save:
        out["G"], out["U"] = host(G), host(U)
    return out


def oracle_layer(cfg, t, w_used):
    r = orc.route(t["X"], t["R"], cfg.T)
    f = orc.ffn_fwd(t["X"], w_used, t["Wg"], t["Wu"], t["Wd"], cfg.T, want_gu=True)
    g = orc.ffn_bwd(t["X"], w_used, t["Wg"], t["Wu"], t["Wd"], t["dY"], cfg.T)
    out = {"w": r["w"], "hbar": r["hbar"], "Y": f["Y"], "G": f["G"], "U": f["U"]}
    out.update(g)
    return out


def compare(cfg, got, ref, names, tol):
    """Whole-tensor rel-L2, worst-row rel-L2 and largest absolute error of every named tensor
    (parity_util.check: the last two are what a single wrong tile or ragged last block trips)."""
    return {k: check(f"{cfg.name} {k}", got[k], ref[k], tol) for k in names}


ALL = ("Y", "G", "U", "dX", "dWg", "dWu", "dWd", "dw")


# ------------------------------------------------------------------ fp32

@pytest.mark.parametrize("structured", [False, True])
def test_c1_fp32_route_fwd_bwd(structured):
    cfg = CONFIGS["C1"]
    t = make_inputs(cfg, structured=structured)
    got = run_layer(cfg, t)
    # the FFN is checked with the GPU's own routing weights as the oracle's input,
    # the routing weights themselves against the oracle's route
    ref = oracle_layer(cfg, t, got["w_used"])
    compare(cfg, got, ref, ("w", "hbar"), 1e-6)
    np.testing.assert_allclose(got["w"].sum(-1), 1.0, atol=1e-6)
    compare(cfg, got, ref, ALL, TOL["f32"])


@pytest.mark.parametrize("cfg", [
    LoryConfig("f32_ragged_dims", B=3, L=60, T=20, d=50, d_ff=70, E=5, dtype="f32", seed=21),
    LoryConfig("f32_single_segment", B=2, L=48, T=48, d=32, d_ff=96, E=3, dtype="f32", seed=22),
    LoryConfig("f32_one_expert", B=1, L=64, T=16, d=24, d_ff=40, E=1, dtype="f32", seed=23),
    LoryConfig("f32_max_experts", B=1, L=32, T=8, d=16, d_ff=24, E=64, dtype="f32", seed=24),
    LoryConfig("f32_one_token_segments", B=2, L=6, T=1, d=12, d_ff=20, E=4, dtype="f32", seed=25),
], ids=lambda c: c.name)
def test_fp32_edge_shapes(cfg):
    t = make_inputs(cfg, structured=True)
    got = run_layer(cfg, t, save=(cfg.E != 1))
    ref = oracle_layer(cfg, t, got["w_used"])
    compare(cfg, got, ref, ("w", "hbar"), 1e-6)
    names = ALL if cfg.E != 1 else ("Y", "dX", "dWg", "dWu", "dWd", "dw")
    compare(cfg, got, ref, names, TOL["f32"])


def test_fp32_given_routing_weights_onehot_and_accumulate():
    cfg = CONFIGS["C1"]
    t = make_inputs(cfg)
    w1 = make_routing_weights(cfg, "onehot")
    got = run_layer(cfg, t, w_override=w1)
    ref = oracle_layer(cfg, t, w1)
    compare(cfg, got, ref, ALL, TOL["f32"])
    # accumulate=1 adds to existing gradient stacks; dX and dw are overwritten
    X, Wg, Wu, Wd, dY = (to_dev(t[k], cfg) for k in ("X", "Wg", "Wu", "Wd", "dY"))
    w = torch.from_numpy(w1).cuda()
    base = [torch.full_like(Wg, 0.5), torch.full_like(Wu, -0.25), torch.full_like(Wd, 2.0)]
    dX, dWg, dWu, dWd, dw = lb.lory_merged_ffn_bwd(X, w, Wg, Wu, Wd, dY, cfg.T, dWg=base[0], dWu=base[1],
                                                   dWd=base[2], accumulate=True)
    torch.cuda.synchronize()
    assert rel_l2(host(dWg) - 0.5, ref["dWg"]) <= 1e-4
    assert rel_l2(host(dWu) + 0.25, ref["dWu"]) <= 1e-4
    assert rel_l2(host(dWd) - 2.0, ref["dWd"]) <= 1e-4
    assert rel_l2(host(dX), ref["dX"]) <= TOL["f32"]
    assert rel_l2(host(dw), ref["dw"]) <= TOL["f32"]


def test_errors_leave_outputs_untouched():
    cfg = CONFIGS["C1"]
    t = make_inputs(cfg)
    X, Wg, Wu, Wd = (to_dev(t[k], cfg) for k in ("X", "Wg", "Wu", "Wd"))
    w = torch.full((cfg.S, cfg.E), 1.0 / cfg.E, device="cuda")
    Y = torch.full_like(X, 7.0)
    tiny_ws = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(lb.LoryError) as ei:
        lb.lory_merged_ffn_fwd(X, w, Wg, Wu, Wd, cfg.T, Y=Y, workspace=tiny_ws)
    assert ei.value.status == lb.LORY_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((Y == 7.0).all())
    # the library stays usable
    lb.lory_merged_ffn_fwd(X, w, Wg, Wu, Wd, cfg.T, Y=Y)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(Y).all()) and not bool((Y == 7.0).all())


# ------------------------------------------------------------------ bf16

BF16_CASES = [
    # (config, slab budget in bytes) - small budgets force several blocks and a ragged last block
    (LoryConfig("bf16_multi_block", B=2, L=512, T=128, d=256, d_ff=576, E=8, dtype="bf16", seed=31), 1 << 20),
    (LoryConfig("bf16_T64", B=2, L=256, T=64, d=128, d_ff=192, E=4, dtype="bf16", seed=32), 256 << 10),
    (LoryConfig("bf16_T256_E32", B=1, L=512, T=256, d=192, d_ff=256, E=32, dtype="bf16", seed=33), 512 << 10),
    (LoryConfig("bf16_E33", B=1, L=256, T=64, d=64, d_ff=128, E=33, dtype="bf16", seed=34), 128 << 20),
    (LoryConfig("bf16_S40", B=5, L=512, T=64, d=64, d_ff=64, E=3, dtype="bf16", seed=35), 128 << 20),
    (LoryConfig("bf16_one_expert", B=1, L=128, T=64, d=64, d_ff=128, E=1, dtype="bf16", seed=36), 128 << 20),
    # segment counts and lengths of the benchmark configurations at reduced widths
    (LoryConfig("bf16_S128_E32", B=8, L=4096, T=256, d=128, d_ff=256, E=32, dtype="bf16", seed=37), 4 << 20),
    (LoryConfig("bf16_S256_T64_E16", B=4, L=4096, T=64, d=128, d_ff=256, E=16, dtype="bf16", seed=38), 128 << 20),
    (LoryConfig("bf16_T1024_E16", B=1, L=2048, T=1024, d=128, d_ff=256, E=16, dtype="bf16", seed=39), 128 << 20),
    (LoryConfig("bf16_S300_E64", B=5, L=3840, T=64, d=64, d_ff=128, E=64, dtype="bf16", seed=40), 128 << 20),
    # 129-256 segments with at most 16 experts: the scatter instance that parks its expert chunks in LDS,
    # here with fewer 16-segment blocks than its static bound
    (LoryConfig("bf16_S160_E12", B=5, L=2048, T=64, d=64, d_ff=128, E=12, dtype="bf16", seed=44), 128 << 20),
    # every GEMM on the persistent ring kernel with two tiles per workgroup (tile boundaries inside
    # the K-step stream), all outputs compared element by element
    (LoryConfig("bf16_ring_two_tiles", B=4, L=4096, T=256, d=512, d_ff=1024, E=4, dtype="bf16", seed=43),
     6144 << 20),
]


@pytest.fixture
def default_budget():
    yield
    lb.lory_set_slab_budget(6144 << 20)


@pytest.mark.parametrize("cfg,budget", BF16_CASES, ids=lambda v: v.name if isinstance(v, LoryConfig) else str(v))
def test_bf16_small_shapes(cfg, budget, default_budget):
    lb.lory_set_slab_budget(budget)
    t = make_inputs(cfg, structured=True)
    got = run_layer(cfg, t)
    ref = oracle_layer(cfg, t, got["w_used"])
    compare(cfg, got, ref, ("w", "hbar"), 1e-5)
    compare(cfg, got, ref, ALL, TOL["bf16"])


def test_bf16_recompute_bf16_grads_and_accumulate(default_budget):
    cfg = BF16_CASES[0][0]
    lb.lory_set_slab_budget(1 << 20)
    t = make_inputs(cfg, structured=True)
    w1 = make_routing_weights(cfg, "peaked")
    # no saved activations: the backward recomputes G and U; gradients stored as bf16
    got = run_layer(cfg, t, w_override=w1, save=False, grad_dtype=torch.bfloat16)
    ref = oracle_layer(cfg, t, w1)
    compare(cfg, got, ref, ("Y", "dX", "dWg", "dWu", "dWd", "dw"), TOL["bf16"])
    X, Wg, Wu, Wd, dY = (to_dev(t[k], cfg) for k in ("X", "Wg", "Wu", "Wd", "dY"))
    w = torch.from_numpy(w1).cuda()
    for gd in (torch.float32, torch.bfloat16):
        base = [torch.full(Wg.shape, 0.5, dtype=gd, device="cuda"),
                torch.full(Wu.shape, -0.25, dtype=gd, device="cuda"),
                torch.full(Wd.shape, 2.0, dtype=gd, device="cuda")]
        lb.lory_merged_ffn_bwd(X, w, Wg, Wu, Wd, dY, cfg.T, dWg=base[0], dWu=base[1], dWd=base[2],
                               accumulate=True, grad_dtype=gd)
        torch.cuda.synchronize()
        for got_sum, c, key in ((base[0], 0.5, "dWg"), (base[1], -0.25, "dWu"), (base[2], 2.0, "dWd")):
            # the increment itself is held to the bf16 bar; a bf16 sum c + dW is stored with one more
            # rounding, uniform within half a bf16 spacing (<= 2^-7 |c + dW|), i.e. an rms error of at
            # most 2^-7 / sqrt(12) of the stored values, measured here against the increment
            rms = lambda a: float(np.sqrt(np.mean(np.square(a))))
            store = (2.0 ** -7 / np.sqrt(12.0)) * rms(ref[key] + c) / rms(ref[key]) if gd == torch.bfloat16 else 0.0
            err = rel_l2(host(got_sum) - c, ref[key])
            print(f"[parity] accumulate {key} {gd}: {err:.2e} (bar {TOL['bf16'] + store:.2e})", flush=True)
            assert err <= TOL["bf16"] + store, (key, gd, err)


def test_bf16_onehot_and_determinism(default_budget):
    cfg = BF16_CASES[0][0]
    lb.lory_set_slab_budget(1 << 20)
    t = make_inputs(cfg)
    w1 = make_routing_weights(cfg, "onehot")
    a = run_layer(cfg, t, w_override=w1)
    b = run_layer(cfg, t, w_override=w1)
    ref = oracle_layer(cfg, t, w1)
    compare(cfg, a, ref, ALL, TOL["bf16"])
    for key in ALL:
        assert np.array_equal(a[key], b[key]), key


@pytest.mark.parametrize("idx", [0, 6])
def test_bf16_saved_merged_parameters_match_remerge(idx, default_budget):
    """The forward may hand its merged parameters to the backward; results are those of the
    re-merging path (same values, same accumulation order), and within tolerance of the oracle."""
    cfg, budget = BF16_CASES[idx]
    lb.lory_set_slab_budget(budget)
    t = make_inputs(cfg, structured=True)
    a = run_layer(cfg, t, merged_save=True)
    b = run_layer(cfg, t, merged_save=False)
    ref = oracle_layer(cfg, t, a["w_used"])
    compare(cfg, a, ref, ALL, TOL["bf16"])
    for key in ALL:
        assert np.array_equal(a[key], b[key]), key


# ------------------------------------------------------------------ merge inside the GEMM

FUSED_CASES = [
    # T = 256: one segment per wavefront; odd number of 64-column blocks, K not a multiple of 64
    LoryConfig("fused_T256", B=2, L=1024, T=256, d=192, d_ff=320, E=8, dtype="bf16", seed=91),
    # T = 128 on the large tile (two segments per wavefront) and on the small one (512 tokens)
    LoryConfig("fused_T128", B=2, L=512, T=128, d=128, d_ff=192, E=32, dtype="bf16", seed=92),
    LoryConfig("fused_T128_small", B=1, L=512, T=128, d=128, d_ff=128, E=5, dtype="bf16", seed=93),
    # T = 64: two segments per wavefront on the small tile; three tasks along the rows
    LoryConfig("fused_T64", B=3, L=512, T=64, d=128, d_ff=256, E=16, dtype="bf16", seed=94),
    # T = 64 on the eight-wave kernel with the second group of eight experts partly and wholly absent
    LoryConfig("fused_T64_E11", B=2, L=256, T=64, d=128, d_ff=192, E=11, dtype="bf16", seed=97),
    LoryConfig("fused_T64_E5", B=1, L=512, T=64, d=64, d_ff=128, E=5, dtype="bf16", seed=98),
    # T = 64 with more than 16 experts: the four-wave kernel, two segments per wavefront
    LoryConfig("fused_T64_E32", B=1, L=512, T=64, d=64, d_ff=128, E=32, dtype="bf16", seed=99),
    LoryConfig("fused_one_expert", B=1, L=1024, T=256, d=64, d_ff=64, E=1, dtype="bf16", seed=95),
    # more tasks than one round of workgroups per XCD block, several K steps per source
    LoryConfig("fused_many_tasks", B=4, L=2048, T=128, d=512, d_ff=1024, E=16, dtype="bf16", seed=96),
]


@pytest.fixture
def fused_everywhere():
    lb.lory_set_fused_merge(2)
    yield
    lb.lory_set_fused_merge(1)


@pytest.mark.parametrize("cfg", FUSED_CASES, ids=lambda c: c.name)
@pytest.mark.parametrize("save", [True, False], ids=["saved_GU", "recompute_GU"])
def test_bf16_fused_merge_gemm(cfg, save, fused_everywhere, default_budget):
    """Token contractions with the merge inside the GEMM (no merged parameter in memory), forward
    and backward, against the oracle; and bit-reproducible."""
    t = make_inputs(cfg, structured=True)
    got = run_layer(cfg, t, save=save, grad_dtype=torch.bfloat16)
    ref = oracle_layer(cfg, t, got["w_used"])
    names = ALL if save else ("Y", "dX", "dWg", "dWu", "dWd", "dw")
    compare(cfg, got, ref, names, TOL["bf16"])
    again = run_layer(cfg, t, save=save, grad_dtype=torch.bfloat16)
    for key in names:
        assert np.array_equal(got[key], again[key]), key


@pytest.fixture
def fused_with_gradients():
    lb.lory_set_fused_merge(3)
    yield
    lb.lory_set_fused_merge(1)


# shapes the expert-gradient kernel takes (at most 16 experts, T a multiple of 64, B L / T a multiple
# of 8); the last one has three tiles along each matrix dimension and experts beyond E in the operand
FSG_CASES = [c for c in FUSED_CASES if c.name in ("fused_T256", "fused_T64", "fused_T64_E11", "fused_T64_E5",
                                                  "fused_many_tasks")]


@pytest.mark.parametrize("cfg", FSG_CASES, ids=lambda c: c.name)
@pytest.mark.parametrize("save", [True, False], ids=["saved_GU", "recompute_GU"])
def test_bf16_fused_expert_gradients(cfg, save, fused_with_gradients, default_budget):
    """As above, and with the per-segment weight gradients kept on chip: expert gradients and
    routing-weight gradients from the kernel that forms X_s^T dG_s; bit-reproducible (every wave adds
    its inner products to a slot of its own, and the slots are summed in a fixed order)."""
    assert cfg.E <= 16 and cfg.T % 64 == 0 and cfg.S % 8 == 0
    t = make_inputs(cfg, structured=True)
    got = run_layer(cfg, t, save=save, grad_dtype=torch.bfloat16)
    ref = oracle_layer(cfg, t, got["w_used"])
    names = ALL if save else ("Y", "dX", "dWg", "dWu", "dWd", "dw")
    compare(cfg, got, ref, names, TOL["bf16"])
    again = run_layer(cfg, t, save=save, grad_dtype=torch.bfloat16)
    for key in names:
        assert np.array_equal(got[key], again[key]), key


def test_bf16_fused_expert_gradients_differ_from_slab_path_only_by_rounding(fused_with_gradients, default_budget):
    """The same call with the slab pipeline for the weight stage (mode 2): the two agree to bf16
    rounding, which shows that mode 3 ran another kernel and that both compute the same thing."""
    cfg = FUSED_CASES[3]
    t = make_inputs(cfg, structured=True)
    on_chip = run_layer(cfg, t, grad_dtype=torch.bfloat16)
    lb.lory_set_fused_merge(2)
    slab = run_layer(cfg, t, grad_dtype=torch.bfloat16)
    for key in ("dWg", "dWu", "dWd", "dw"):
        check(f"{cfg.name} {key} on chip vs slab", on_chip[key], slab[key], TOL["bf16"])
    assert any(not np.array_equal(on_chip[k], slab[k]) for k in ("dWg", "dWu", "dWd"))


def test_bf16_fused_onehot_routing(fused_everywhere):
    """One-hot routing weights select exactly one expert: the fused kernel's merged tiles are then
    copies of that expert's (bf16 values pass through the hi + lo weight pair unchanged)."""
    cfg = FUSED_CASES[3]
    t = make_inputs(cfg)
    w1 = make_routing_weights(cfg, "onehot")
    got = run_layer(cfg, t, w_override=w1)
    ref = oracle_layer(cfg, t, w1)
    compare(cfg, got, ref, ALL, TOL["bf16"])


def test_merged_save_unsupported_shapes_are_rejected():
    shape = lb.make_shape(5, 3840, 64, 64, 128, 64, torch.bfloat16)   # S = 300 > 128 at E = 64
    assert lb.lory_merged_save_bytes(shape) == 0
    shape32 = lb.make_shape(2, 512, 128, 64, 256, 4, torch.float32)
    assert lb.lory_merged_save_bytes(shape32) == 0


# ------------------------------------------------------------------ router backward

ROUTE_BWD_CASES = [
    CONFIGS["C1"],
    LoryConfig("f32_ragged_dims", B=3, L=60, T=20, d=50, d_ff=70, E=5, dtype="f32", seed=21),
    LoryConfig("f32_single_segment", B=2, L=48, T=48, d=32, d_ff=96, E=3, dtype="f32", seed=22),
    LoryConfig("f32_max_experts", B=1, L=32, T=8, d=16, d_ff=24, E=64, dtype="f32", seed=24),
    LoryConfig("f32_one_token_segments", B=2, L=6, T=1, d=12, d_ff=20, E=4, dtype="f32", seed=25),
    LoryConfig("f32_many_segments", B=2, L=640, T=4, d=40, d_ff=8, E=6, dtype="f32", seed=26),
    LoryConfig("bf16_route_bwd", B=2, L=512, T=64, d=192, d_ff=64, E=8, dtype="bf16", seed=41),
    LoryConfig("bf16_route_bwd_E33", B=3, L=384, T=128, d=320, d_ff=64, E=33, dtype="bf16", seed=42),
]


@pytest.mark.parametrize("cfg", ROUTE_BWD_CASES, ids=lambda c: c.name)
def test_route_bwd_matches_oracle(cfg):
    """lory_route_bwd against the oracle's router backward, fed the same dw.

    The routing here is peaked (structured inputs) so that the softmax Jacobian is far from
    degenerate; dw is a seeded N(0,1) tensor, not the FFN's, so that the router path is not small.
    """
    print(f"[gpu] route_bwd {cfg}", flush=True)
    t = make_inputs(cfg, structured=True)
    rng = np.random.Generator(np.random.Philox(cfg.seed + 900))
    dw = rng.standard_normal((cfg.S, cfg.E)).astype(np.float32)
    X, R = to_dev(t["X"], cfg), to_dev(t["R"], cfg)
    hbar = torch.empty((cfg.S, cfg.d), dtype=torch.float32, device="cuda")
    w = lb.lory_route(X, R, cfg.T, hbar=hbar, d_ff=cfg.d_ff)
    dw_d = torch.from_numpy(dw).cuda()
    # (1) router path alone: added to zeros
    dX0 = torch.zeros_like(X)
    dR = lb.lory_route_bwd(R, w, hbar, dw_d, dX0, cfg.T, d_ff=cfg.d_ff)
    # (2) added in place to an existing gradient, dR accumulated on top of the first result
    base = to_dev(t["dY"], cfg)
    dX1 = base.clone()
    dR2 = dR.clone()
    lb.lory_route_bwd(R, w, hbar, dw_d, dX1, cfg.T, dR=dR2, accumulate_dR=True, d_ff=cfg.d_ff)
    torch.cuda.synchronize()
    ref = orc.route_bwd(t["X"], t["R"], dw.astype(np.float64), cfg.T)
    tol = 1e-4 if cfg.dtype == "f32" else TOL["bf16"]   # fp32: forward softmax and means are fp32
    if cfg.N == 1:
        assert not ref["dX_add"].any() and not ref["dR"].any()
        assert not host(dX0).any() and not host(dR).any()
        assert torch.equal(dX1, base)
        return
    got = {"dX_add": host(dX0), "dR": host(dR)}
    compare(cfg, got, ref, ("dX_add", "dR"), tol)
    total = host(base) + ref["dX_add"].reshape(host(base).shape)
    compare(cfg, {"dX_total": host(dX1)}, {"dX_total": total}, ("dX_total",), tol)
    np.testing.assert_array_equal(host(dR2), 2.0 * host(dR))
    # rows of the last segment of every sequence get nothing from the router path
    last = host(dX0).reshape(cfg.B, cfg.N, cfg.T, cfg.d)[:, -1]
    assert not last.any()


def test_whole_layer_gradient_fp32():
    """route -> fwd -> bwd -> route_bwd on the GPU against the oracle's whole-layer gradient."""
    cfg = CONFIGS["C1"]
    t = make_inputs(cfg, structured=True)
    X, R = to_dev(t["X"], cfg), to_dev(t["R"], cfg)
    Wg, Wu, Wd = (to_dev(t[k], cfg) for k in ("Wg", "Wu", "Wd"))
    dY = to_dev(t["dY"], cfg)
    hbar = torch.empty((cfg.S, cfg.d), dtype=torch.float32, device="cuda")
    w = lb.lory_route(X, R, cfg.T, hbar=hbar, d_ff=cfg.d_ff)
    lb.lory_merged_ffn_fwd(X, w, Wg, Wu, Wd, cfg.T)
    dX, dWg, dWu, dWd, dw = lb.lory_merged_ffn_bwd(X, w, Wg, Wu, Wd, dY, cfg.T)
    dR = lb.lory_route_bwd(R, w, hbar, dw, dX, cfg.T, d_ff=cfg.d_ff)
    torch.cuda.synchronize()
    ref = orc.layer_bwd(t["X"], t["R"], t["Wg"], t["Wu"], t["Wd"], t["dY"], cfg.T)
    got = {"dX": host(dX), "dR": host(dR), "dWg": host(dWg), "dWu": host(dWu), "dWd": host(dWd)}
    compare(cfg, got, ref, ("dX", "dWg", "dWu", "dWd"), 2e-5)
    compare(cfg, got, ref, ("dR",), DR_TOL["f32"])
    assert np.linalg.norm(ref["dR"]) > 0


# ------------------------------------------------------------------ inference: prompt-only routing

INFER_CASES = [
    # (config of the expert stacks, prompt length, token counts of the generation-phase calls)
    (LoryConfig("inf_f32", B=3, L=40, T=40, d=48, d_ff=72, E=5, dtype="f32", seed=51), 40, (1, 3, 8, 13)),
    (LoryConfig("inf_f32_odd", B=2, L=7, T=7, d=50, d_ff=70, E=4, dtype="f32", seed=52), 7, (1, 9)),
    (LoryConfig("inf_bf16", B=4, L=200, T=200, d=256, d_ff=704, E=8, dtype="bf16", seed=53), 200,
     (1, 2, 8, 11, 64, 192)),
    (LoryConfig("inf_bf16_wide", B=2, L=96, T=96, d=1024, d_ff=2816, E=32, dtype="bf16", seed=54), 96,
     (1, 5, 256)),
    # prompts long enough for the two-stage mean (vector and scalar column paths)
    (LoryConfig("inf_bf16_long", B=3, L=1000, T=1000, d=256, d_ff=320, E=16, dtype="bf16", seed=58), 1000, (1, 4)),
    (LoryConfig("inf_f32_long_odd", B=2, L=300, T=300, d=50, d_ff=36, E=3, dtype="f32", seed=59), 300, (2,)),
]


@pytest.mark.parametrize("cfg,Lp,steps", INFER_CASES, ids=lambda v: v.name if isinstance(v, LoryConfig) else None)
def test_prompt_only_routing_inference(cfg, Lp, steps):
    """lory_prompt_merge + lory_dense_ffn_fwd against the oracle: routing on the mean of the whole
    prompt (route with T = L), merged parameters by the definition, then the merged FFN on new tokens
    (the oracle's ffn_fwd with one segment per sequence and the same routing weights)."""
    print(f"[gpu] infer {cfg}", flush=True)
    t = make_inputs(cfg, structured=True, with_dy=False)
    tol = TOL[cfg.dtype]
    X, R = to_dev(t["X"], cfg), to_dev(t["R"], cfg)
    Wg, Wu, Wd = (to_dev(t[k], cfg) for k in ("Wg", "Wu", "Wd"))
    w, Wbar = lb.lory_prompt_merge(X, R, Wg, Wu, Wd)
    torch.cuda.synchronize()
    ref_w = orc.route(t["X"], t["R"], Lp)["w"]
    got_w = host(w)
    assert rel_l2(got_w, ref_w) <= 1e-5
    # merged parameters against the definition, from the GPU's own routing weights
    D = cfg.d * cfg.d_ff
    Wb = host(Wbar).reshape(3, cfg.B, D)
    for i, k in enumerate(("Wg", "Wu", "Wd")):
        ref = np.einsum("be,en->bn", got_w, t[k].astype(np.float64).reshape(cfg.E, D))
        err = rel_l2(Wb[i], ref)
        print(f"[parity] {cfg.name}: {k}_bar={err:.2e}", flush=True)
        assert err <= (1e-5 if cfg.dtype == "f32" else 4e-3)
    # generation phase: new tokens of several counts, the same merged parameters
    for n_tok in steps:
        rng = np.random.Generator(np.random.Philox(cfg.seed * 1000 + n_tok))
        Xn_host = rng.standard_normal((cfg.B, n_tok, cfg.d)).astype(np.float32)
        if cfg.dtype == "bf16":
            Xn_host = round_to_bf16(Xn_host)
        Xn = to_dev(Xn_host, cfg)
        Y = lb.lory_dense_ffn_fwd(Xn, Wbar, cfg.d_ff)
        torch.cuda.synchronize()
        ref = orc.ffn_fwd(Xn_host, got_w, t["Wg"], t["Wu"], t["Wd"], n_tok)["Y"]
        err = rel_l2(host(Y), ref)
        print(f"[parity] {cfg.name}: {n_tok} tokens Y={err:.2e}", flush=True)
        assert np.isfinite(err) and err <= tol, (cfg.name, n_tok, err)


def test_prefill_with_saved_merged_parameters_feeds_decode(default_budget):
    """lory_merged_ffn_fwd with T = L and Wbar_save leaves the same buffer lory_prompt_merge writes."""
    cfg = LoryConfig("inf_prefill", B=2, L=128, T=128, d=128, d_ff=256, E=8, dtype="bf16", seed=55)
    t = make_inputs(cfg, structured=True, with_dy=False)
    X, R = to_dev(t["X"], cfg), to_dev(t["R"], cfg)
    Wg, Wu, Wd = (to_dev(t[k], cfg) for k in ("Wg", "Wu", "Wd"))
    w, Wbar = lb.lory_prompt_merge(X, R, Wg, Wu, Wd)
    w2 = lb.lory_route(X, R, cfg.T, d_ff=cfg.d_ff)
    save = lb.alloc_merged_save(lb.make_shape(cfg.B, cfg.L, cfg.T, cfg.d, cfg.d_ff, cfg.E, X.dtype))
    Y = lb.lory_merged_ffn_fwd(X, w2, Wg, Wu, Wd, cfg.T, Wbar_save=save)
    Yd = lb.lory_dense_ffn_fwd(X, Wbar, cfg.d_ff)
    torch.cuda.synchronize()
    assert torch.equal(w, w2)
    assert torch.equal(save.view(torch.bfloat16), Wbar.reshape(-1))
    assert rel_l2(host(Yd), host(Y)) <= 2e-3   # same GEMM kernels; SwiGLU fused against separate pass


def test_prefix_routing_variant():
    """The paper's prefix-routing ablation (Section 5.1): every segment of a sequence uses the merged
    FFN chosen from the first segment.  On the GPU that is lory_prompt_merge on the first T tokens and
    lory_dense_ffn_fwd over the whole sequence; the oracle is its ffn_fwd with the first segment's
    routing weights repeated for every segment."""
    cfg = LoryConfig("prefix", B=2, L=512, T=128, d=128, d_ff=320, E=8, dtype="bf16", seed=56)
    t = make_inputs(cfg, structured=True, with_dy=False)
    X, R = to_dev(t["X"], cfg), to_dev(t["R"], cfg)
    Wg, Wu, Wd = (to_dev(t[k], cfg) for k in ("Wg", "Wu", "Wd"))
    w, Wbar = lb.lory_prompt_merge(X[:, :cfg.T].contiguous(), R, Wg, Wu, Wd)
    Y = lb.lory_dense_ffn_fwd(X, Wbar, cfg.d_ff)
    torch.cuda.synchronize()
    e0 = orc.route(t["X"][:, :cfg.T], t["R"], cfg.T)["w"]            # [B, E]: first segment on itself
    assert rel_l2(host(w), e0) <= 1e-5
    w_rep = np.repeat(host(w), cfg.N, axis=0)                         # the same row for all N segments
    ref = orc.ffn_fwd(t["X"], w_rep, t["Wg"], t["Wu"], t["Wd"], cfg.T)["Y"]
    err = rel_l2(host(Y), ref)
    print(f"[parity] prefix routing Y={err:.2e}", flush=True)
    assert err <= TOL["bf16"]


def test_step_replayed_from_a_hip_graph_matches_eager(default_budget):
    """bench.py times a captured graph of the step; every replay must reproduce the eager results
    bit for bit (the library enqueues kernels only: no allocation, no synchronisation, no memsets)."""
    cfg = LoryConfig("graph", B=2, L=512, T=128, d=256, d_ff=512, E=8, dtype="bf16", seed=61)
    t = make_inputs(cfg, structured=True)
    X, R = to_dev(t["X"], cfg), to_dev(t["R"], cfg)
    Wg, Wu, Wd = (to_dev(t[k], cfg) for k in ("Wg", "Wu", "Wd"))
    dY = to_dev(t["dY"], cfg)
    shape = lb.make_shape(cfg.B, cfg.L, cfg.T, cfg.d, cfg.d_ff, cfg.E, X.dtype)
    ws_f, ws_b = lb.alloc_workspace(shape, lb.LORY_PASS_FWD), lb.alloc_workspace(shape, lb.LORY_PASS_BWD)
    w = torch.empty((cfg.S, cfg.E), dtype=torch.float32, device="cuda")
    hbar = torch.empty((cfg.S, cfg.d), dtype=torch.float32, device="cuda")
    G = torch.empty((cfg.tokens, cfg.d_ff), dtype=X.dtype, device="cuda")
    U = torch.empty_like(G)
    Wbar = lb.alloc_merged_save(shape)
    Y, dX = torch.empty_like(X), torch.empty_like(X)
    dWg, dWu, dWd = torch.empty_like(Wg), torch.empty_like(Wu), torch.empty_like(Wd)
    dw = torch.empty_like(w)
    dR = torch.empty((cfg.d, cfg.E), dtype=torch.float32, device="cuda")
    outs = (w, hbar, Y, dX, dWg, dWu, dWd, dw, dR)

    def step():
        lb.lory_route(X, R, cfg.T, w=w, hbar=hbar, d_ff=cfg.d_ff)
        lb.lory_merged_ffn_fwd(X, w, Wg, Wu, Wd, cfg.T, Y=Y, G_save=G, U_save=U, workspace=ws_f, Wbar_save=Wbar)
        lb.lory_merged_ffn_bwd(X, w, Wg, Wu, Wd, dY, cfg.T, G_save=G, U_save=U, dX=dX, dWg=dWg, dWu=dWu,
                               dWd=dWd, dw=dw, grad_dtype=X.dtype, workspace=ws_b, Wbar_save=Wbar)
        lb.lory_route_bwd(R, w, hbar, dw, dX, cfg.T, dR=dR, d_ff=cfg.d_ff)

    step()
    torch.cuda.synchronize()
    eager = [o.clone() for o in outs]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        for o in outs:
            o.fill_(float("nan")) if o.dtype.is_floating_point else o.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for o, ref in zip(outs, eager):
            assert torch.equal(o, ref), rep
        step()                      # eager work between replays
        torch.cuda.synchronize()


@pytest.mark.parametrize("cfg", [
    CONFIGS["C1"],
    LoryConfig("autograd_bf16", B=2, L=512, T=128, d=256, d_ff=512, E=8, dtype="bf16", seed=71),
], ids=lambda c: c.name)
def test_autograd_wrapper_matches_oracle_layer_gradient(cfg):
    """paper_2405_03133_amd.autograd.lory_layer under torch.autograd against the oracle's whole-layer
    gradient (FFN path + router path with the stop gradient on the first segment)."""
    from paper_2405_03133_amd.autograd import lory_layer
    t = make_inputs(cfg, structured=True)
    leaves = {k: to_dev(t[k], cfg).requires_grad_(True) for k in ("X", "R", "Wg", "Wu", "Wd")}
    dY = to_dev(t["dY"], cfg)
    y = lory_layer(leaves["X"], leaves["R"], leaves["Wg"], leaves["Wu"], leaves["Wd"], cfg.T)
    (y.float() * dY.float()).sum().backward()
    torch.cuda.synchronize()
    ref = orc.layer_bwd(t["X"], t["R"], t["Wg"], t["Wu"], t["Wd"], t["dY"], cfg.T)
    ref_y = orc.layer_fwd(t["X"], t["R"], t["Wg"], t["Wu"], t["Wd"], cfg.T)["Y"]
    tol = 2e-5 if cfg.dtype == "f32" else TOL["bf16"]
    got = {"Y": host(y), "dX": host(leaves["X"].grad), "dWg": host(leaves["Wg"].grad),
           "dWu": host(leaves["Wu"].grad), "dWd": host(leaves["Wd"].grad), "dR": host(leaves["R"].grad)}
    ref = dict(ref, Y=ref_y)
    compare(cfg, got, ref, ("Y", "dX", "dWg", "dWu", "dWd"), tol)
    compare(cfg, got, ref, ("dR",), DR_TOL[cfg.dtype])


@pytest.mark.parametrize("L,lens", [(96, [96, 1, 37, 64]), (512, [512, 1, 300, 257])], ids=["short", "long"])
def test_prompt_merge_with_prompts_of_different_lengths(L, lens):
    """Padded prompts with a length per sequence: routing on the mean of the first len[b] rows only
    (the oracle routes each sequence on its own, with T = L = len[b]); padding rows hold NaN."""
    cfg = LoryConfig("inf_ragged", B=4, L=L, T=L, d=128, d_ff=192, E=8, dtype="bf16", seed=57)
    t = make_inputs(cfg, structured=True, with_dy=False)
    lens = np.array(lens, dtype=np.int32)
    Xp = t["X"].copy()
    for b, n in enumerate(lens):
        Xp[b, n:] = np.nan
    X, R = to_dev(Xp, cfg), to_dev(t["R"], cfg)
    Wg, Wu, Wd = (to_dev(t[k], cfg) for k in ("Wg", "Wu", "Wd"))
    w, Wbar = lb.lory_prompt_merge(X, R, Wg, Wu, Wd, prompt_len=torch.from_numpy(lens).cuda())
    torch.cuda.synchronize()
    got_w = host(w)
    assert np.isfinite(got_w).all() and torch.isfinite(Wbar.float()).all()
    for b, n in enumerate(lens):
        ref = orc.route(t["X"][b:b + 1, :n], t["R"], int(n))["w"][0]
        assert rel_l2(got_w[b], ref) <= 1e-5, (b, n)
    D = cfg.d * cfg.d_ff
    ref_g = np.einsum("be,en->bn", got_w, t["Wg"].astype(np.float64).reshape(cfg.E, D))
    assert rel_l2(host(Wbar).reshape(3, cfg.B, D)[0], ref_g) <= 4e-3
