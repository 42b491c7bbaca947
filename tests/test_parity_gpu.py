"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU
oracle on the same seeded inputs, element by element.

Bar: max|Y - Yref| / max|Yref| <= 2e-2 for bf16 inputs with fp32 accumulation (2e-3 for IEEE half),
<= 1e-5 in the fp32 test mode.
"""
import numpy as np
import pytest
import torch

import dfk_inputs as di
import paper_2602_11808_amd as dfk
from oracle import oracle
from tests.helpers import TOL_BF16, TOL_FP16, TOL_FP32, assert_parity, rel_err

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _dt(dtype):
    return {"bf16": dfk.DFK_BF16, "fp32": dfk.DFK_FP32, "fp16": dfk.DFK_FP16}[dtype]


def _tol(dtype):
    return {"bf16": TOL_BF16, "fp32": TOL_FP32, "fp16": TOL_FP16}[dtype]


def gpu_inputs(t):
    return {k: di.to_torch(v, DEV) for k, v in t.items()}


def run_ex(g, cfg, ws=None):
    M, d = g["X"].shape
    ff = g["Wg"].shape[0]
    if ws is None:
        ws = dfk.new_workspace(M, d, ff, DEV)
    Y = torch.full_like(g["X"], float("nan"))
    dfk.dfk_swiglu_mlp_ex(g["X"], g["Wg"], g["Wu"], g["Wd"], Y, cfg, ws)
    torch.cuda.synchronize()
    return Y, ws


def y64(Y):
    return di.as_f64(di.to_numpy(Y))


def workspace_is_clean(ws, M, d):
    """Arrival counters and the atomic accumulator must be zero again after a call."""
    head = ws[:4096 + 64 * 32768 * 4]
    return int(torch.count_nonzero(head).item()) == 0


SMALL = [
    # (M, d_model, d_ff): the tiny configuration, ragged tails, several slices
    (1, 512, 1536),
    (1, 8, 8),
    (2, 264, 1000),
    (3, 1024, 2056),
    (5, 520, 4104),
    (8, 512, 1536),
    (9, 256, 520),
    (16, 512, 1536),
    (17, 128, 264),
]


@pytest.mark.parametrize("dtype", ["bf16", "fp32", "fp16"])
@pytest.mark.parametrize("shape", SMALL, ids=lambda s: "M%d_d%d_ff%d" % s)
def test_every_candidate_matches_oracle_small(shape, dtype):
    M, d, ff = shape
    t = di.mlp_inputs(M, d, ff, seed=0, dtype=dtype)
    ref = oracle.swiglu_mlp(t["X"], t["Wg"], t["Wu"], t["Wd"])
    g = gpu_inputs(t)
    n = dfk.dfk_num_candidates(M, d, ff, _dt(dtype))
    assert n > 0
    ws = None
    seen = set()
    for i in range(n):
        cfg = dfk.dfk_get_candidate(M, d, ff, _dt(dtype), i)
        print("case", shape, dtype, cfg, flush=True)
        Y, ws = run_ex(g, cfg, ws)
        assert_parity(y64(Y), ref, dtype, (shape, dtype, cfg))
        assert workspace_is_clean(ws, M, d), (shape, dtype, cfg)
        seen.add((cfg.variant, cfg.path))
    assert any(v == dfk.DFK_VARIANT_FUSED for v, _ in seen)
    assert any(v == dfk.DFK_VARIANT_TWO_KERNEL for v, _ in seen)


def test_tiny_config_against_stored_oracle_output():
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "c1_tiny_y.txt")
    want = np.array([float.fromhex(l) for l in open(path) if not l.startswith("#")])[None]
    g = gpu_inputs(di.mlp_inputs(1, 512, 1536, seed=0))
    ws = dfk.new_workspace(1, 512, 1536, DEV)
    dfk.dfk_set_workspace(ws)
    for fn in (dfk.dfk_swiglu_mlp, dfk.dfk_swiglu_mlp_fused, dfk.dfk_swiglu_mlp_unfused):
        Y = torch.empty_like(g["X"])
        fn(g["X"], g["Wg"], g["Wu"], g["Wd"], Y)
        torch.cuda.synchronize()
        assert rel_err(y64(Y), want) <= TOL_BF16, fn.__name__
    dfk.dfk_set_workspace(None)


FULL = [
    # the configurations the benchmark times, at their real sizes
    ("llama3-8b", 4096, 14336, (1, 2, 4, 8, 16, 64, 256)),
    ("qwen2.5-32b", 5120, 27648, (1, 8, 32, 64)),
    ("llama3-70b", 8192, 28672, (1, 16, 64, 128)),
]


@pytest.mark.parametrize("name,d,ff,Ms", FULL, ids=[f[0] for f in FULL])
def test_full_size_entry_points_match_oracle(name, d, ff, Ms):
    """Default entry points (scheduler's choice, forced fused, forced two-kernel)
    at full size, in the launch configuration the benchmark uses.  Up to 16 tokens every
    output is compared; beyond, the rows of a sample of tokens (rows of Y are independent,
    so the oracle computes exactly those)."""
    Mmax = max(Ms)
    g = di.mlp_inputs_torch(Mmax, d, ff, seed=0, device=DEV)
    host = {k: di.to_numpy(v) for k, v in g.items()}
    ws = dfk.new_workspace(Mmax, d, ff, DEV)
    dfk.dfk_set_workspace(ws)
    try:
        for M in Ms:
            X = g["X"][:M].contiguous()
            rows = list(range(M)) if M <= 16 else sorted({0, 1, 15, 16, M // 2, M - 2, M - 1})
            ref = oracle.swiglu_mlp(host["X"][rows], host["Wg"], host["Wu"], host["Wd"])
            assert 0.05 < np.abs(ref).max() < 50.0
            fns = (dfk.dfk_swiglu_mlp, dfk.dfk_swiglu_mlp_fused, dfk.dfk_swiglu_mlp_unfused)
            for fn in fns:   # beyond its tokens per launch the fused form runs as several launches
                print("case", name, "M", M, fn.__name__, flush=True)
                Y = torch.full_like(X, float("nan"))
                fn(X, g["Wg"], g["Wu"], g["Wd"], Y)
                torch.cuda.synchronize()
                assert bool(torch.isfinite(Y.float()).all()), (name, M, fn.__name__)
                assert_parity(y64(Y)[rows], ref, "bf16", (name, M, fn.__name__))
                assert workspace_is_clean(ws, M, d)
    finally:
        dfk.dfk_set_workspace(None)


@pytest.mark.parametrize("M", [33, 64, 100, 256])
def test_large_token_counts(M):
    d, ff = 1024, 2816
    t = di.mlp_inputs(M, d, ff, seed=3)
    ref = oracle.swiglu_mlp(t["X"], t["Wg"], t["Wu"], t["Wd"])
    g = gpu_inputs(t)
    ws = dfk.new_workspace(M, d, ff, DEV)
    for variant in (dfk.DFK_VARIANT_FUSED, dfk.DFK_VARIANT_TWO_KERNEL):
        for i in range(dfk.dfk_num_candidates(M, d, ff, dfk.DFK_BF16)):
            cfg = dfk.dfk_get_candidate(M, d, ff, dfk.DFK_BF16, i)
            if cfg.variant != variant:
                continue
            print("case M", M, cfg, flush=True)
            Y, _ = run_ex(g, cfg, ws)
            assert_parity(y64(Y), ref, "bf16", (M, cfg))
            assert workspace_is_clean(ws, M, d)
            break


@pytest.mark.parametrize("shape", [(1, 1024, 2816), (16, 1024, 4104), (17, 1024, 2816), (33, 2048, 4104),
                                   (48, 1024, 2816), (64, 1024, 8200), (100, 1024, 2816),
                                   (3, 768, 1000), (40, 1280, 2056), (64, 2304, 1536), (16, 896, 1000), (33, 640, 520),
                                   (5, 512, 40968)],
                         ids=lambda s: "M%d_d%d_ff%d" % s)
def test_kernels_for_up_to_64_tokens_per_launch(shape):
    """Every candidate of the kernels whose activations travel through the tile rings (config field
    kmajor = 1: the pair for up to 64 tokens per launch, and the single launch built on its stage one; kmajor = 3:
    beyond 32 tokens, the gate/up kernel with workgroup-shared weight tiles in front of the same down kernel;
    kmajor = 4: both kernels' workgroups in one launch, the down workgroups waiting for the gate/up workgroups of
    their rows):
    one to four token tiles, ragged d_ff, both reductions, and a token count that needs two launches; the last five shapes have a d_model whose 128-k chunks do not
    divide evenly among the wavefronts (6, 10, 18, 7 and 5 chunks for 4 or 8 wavefronts); the last one a d_ff
    beyond 512 slices of 64 rows, which runs with more slices."""
    M, d, ff = shape
    t = di.mlp_inputs(M, d, ff, seed=11)
    ref = oracle.swiglu_mlp(t["X"], t["Wg"], t["Wu"], t["Wd"])
    g = gpu_inputs(t)
    ws = dfk.new_workspace(M, d, ff, DEV)
    cfgs = _cfgs(M, d, ff, lambda c: c.kmajor in (1, 3, 4))
    assert any(c.kmajor == 4 for c in cfgs) == (d // 128 >= 8)
    assert cfgs
    assert {c.reduce for c in cfgs} == {dfk.DFK_REDUCE_TICKET, dfk.DFK_REDUCE_ATOMIC}
    assert any(c.kmajor == 3 for c in cfgs) == (M > 32 and d // 128 >= 8)   # its down kernel runs eight wavefronts
    for cfg in cfgs:
        print("case", shape, cfg, flush=True)
        for _ in range(2):
            Y, _ = run_ex(g, cfg, ws)
            assert_parity(y64(Y), ref, "bf16", (shape, cfg))
            assert workspace_is_clean(ws, M, d), (shape, cfg)


@pytest.mark.parametrize("dtype", ["bf16", "fp16"])
@pytest.mark.parametrize("shape", [(65, 1024, 2816), (100, 512, 1000), (128, 1024, 4104), (129, 2048, 4104),
                                   (200, 512, 1536), (256, 1024, 4104), (130, 128, 264), (256, 256, 520), (256, 512, 8200),
                                   (3, 384, 1000), (40, 256, 2056), (64, 384, 1536), (70, 512, 33000)],
                         ids=lambda s: "M%d_d%d_ff%d" % s)
def test_kernels_for_up_to_256_tokens_per_launch(shape, dtype):
    """Every candidate of the pair of kernels whose workgroups share the weight tiles (config
    field kmajor = 2): two and four token tiles per wavefront, token tiles that are partly or
    wholly empty, ragged d_ff, both reductions, up to the largest token count a call accepts; the
    two shapes before the last have fewer pipeline steps than buffers (one or two k chunks, 8-row d_ff splits);
    in (256, 512, 8200) A_2 is larger than one L2, where the down kernel places the workgroups of a split on one
    XCD; the last three are token counts of 64 and below at a d_model the 64-token pair cannot take (fewer
    128-k chunks than wavefronts), where this pair is offered instead; the last one a d_ff beyond 512 slices of
    64 rows."""
    M, d, ff = shape
    t = di.mlp_inputs(M, d, ff, seed=29, dtype=dtype)
    ref = oracle.swiglu_mlp(t["X"], t["Wg"], t["Wu"], t["Wd"])
    g = gpu_inputs(t)
    ws = dfk.new_workspace(M, d, ff, DEV)
    n = dfk.dfk_num_candidates(M, d, ff, _dt(dtype))
    cfgs = [c for c in (dfk.dfk_get_candidate(M, d, ff, _dt(dtype), i) for i in range(n)) if c.kmajor == 2]
    assert cfgs
    assert {c.reduce for c in cfgs} == {dfk.DFK_REDUCE_TICKET, dfk.DFK_REDUCE_ATOMIC}
    for cfg in cfgs:
        print("case", shape, dtype, cfg, flush=True)
        for _ in range(2):
            Y, _ = run_ex(g, cfg, ws)
            assert_parity(y64(Y), ref, dtype, (shape, cfg))
            assert workspace_is_clean(ws, M, d), (shape, cfg)


@pytest.mark.parametrize("d,ff,Ms", [(4096, 14336, (128, 256)), (5120, 27648, (128,)), (8192, 8200, (256,))],
                         ids=["llama3_8b", "qwen2.5_32b", "wide_d8192"])
def test_kernels_for_up_to_256_tokens_full_size_sampled_rows(d, ff, Ms):
    """Full-size layers at 128 and 256 tokens in one launch: a sample of tokens against the oracle
    (the second shape has 40 column blocks and d_ff slices of 6 and 7 row tiles; the third 64 column blocks,
    so the down kernel runs with 4 and 8 d_ff splits).  Between them the three ways the down kernel maps
    workgroups to (split, column block) when A_2 exceeds one L2: splits a multiple of 8, splits dividing 8,
    and the plain order for anything else (6 and 12 splits)."""
    g = di.mlp_inputs_torch(max(Ms), d, ff, seed=31, device=DEV)
    host = {k: di.to_numpy(v) for k, v in g.items()}
    ws = dfk.new_workspace(max(Ms), d, ff, DEV)
    for M in Ms:
        X = g["X"][:M].contiguous()
        rows = sorted({0, 17, 63, 64, M // 2 + 5, M - 16, M - 1})
        ref = oracle.swiglu_mlp(host["X"][rows], host["Wg"], host["Wu"], host["Wd"])
        cfgs = [c for c in _cfgs(M, d, ff, lambda c: c.kmajor == 2)]
        picked = {}   # the first candidate of each (reduction, number of d_ff splits of the down kernel)
        for c in cfgs:
            picked.setdefault((c.reduce, c.k2_splits), c)
        assert {r for r, _ in picked} == {dfk.DFK_REDUCE_TICKET, dfk.DFK_REDUCE_ATOMIC}
        picked = list(picked.values())
        for cfg in picked:
            print("case full", M, cfg, flush=True)
            Y = torch.full_like(X, float("nan"))
            dfk.dfk_swiglu_mlp_ex(X, g["Wg"], g["Wu"], g["Wd"], Y, cfg, ws)
            torch.cuda.synchronize()
            assert bool(torch.isfinite(Y.float()).all()), (M, cfg)
            assert_parity(y64(Y)[rows], ref, "bf16", (M, cfg))
            assert workspace_is_clean(ws, M, d)


def _block_case(M, d, ff, dtype, seed):
    t = di.mlp_inputs(M, d, ff, seed=seed, dtype=dtype)
    t["w"] = di.tensor(seed + 1000, (d,), 1.0, dtype)
    return t


@pytest.mark.parametrize("dtype", ["bf16", "fp16"])
@pytest.mark.parametrize("shape", [(1, 1024, 2816), (5, 512, 1000), (16, 1024, 4104), (17, 1024, 2816), (33, 2048, 4104),
                                   (64, 1024, 8200), (70, 1024, 2816), (130, 512, 1536), (256, 1024, 2816), (9, 768, 1000), (20, 384, 520)],
                         ids=lambda s: "M%d_d%d_ff%d" % s)
def test_mlp_block_with_norm_and_residual(shape, dtype):
    """H + MLP(RMSNorm(H)) in the two launches of the plain block, against the oracle's
    composition: every candidate of the kernel pair that carries it, both reductions, one to
    four token tiles and several launches, out of place and in place."""
    M, d, ff = shape
    eps = 1e-5
    t = _block_case(M, d, ff, dtype, seed=17)
    ref = oracle.mlp_block(t["X"], t["w"], eps, t["Wg"], t["Wu"], t["Wd"])
    H64 = di.as_f64(t["X"])
    g = gpu_inputs(t)
    ws = dfk.new_workspace(M, d, ff, DEV)
    n = dfk.dfk_num_candidates(M, d, ff, _dt(dtype))
    every = [dfk.dfk_get_candidate(M, d, ff, _dt(dtype), i) for i in range(n)]
    # the two kernel pairs that carry this form (the 256-token pair with the normalisation as a launch of its
    # own ahead of it); anything else is refused
    cfgs = [c for c in every if c.kmajor in (1, 2) and c.variant == dfk.DFK_VARIANT_TWO_KERNEL]
    assert {c.reduce for c in cfgs} == {dfk.DFK_REDUCE_TICKET, dfk.DFK_REDUCE_ATOMIC}
    assert any(c.kmajor == 2 for c in cfgs) == (M > 64 or d < 512)
    for c in [c for c in every if c not in cfgs][:3]:
        with pytest.raises(dfk.DfkError) as ei:
            dfk.dfk_mlp_block(g["X"], g["w"], eps, g["Wg"], g["Wu"], g["Wd"], torch.empty_like(g["X"]), c, ws)
        assert ei.value.status == dfk.DFK_ERR_UNSUPPORTED_SHAPE
    tol = _tol(dtype)
    for cfg in cfgs:
        print("case", shape, dtype, cfg, flush=True)
        out = torch.full_like(g["X"], float("nan"))
        dfk.dfk_mlp_block(g["X"], g["w"], eps, g["Wg"], g["Wu"], g["Wd"], out, cfg, ws)
        torch.cuda.synchronize()
        got = y64(out)
        assert_parity(got, ref, dtype, (shape, cfg))
        # the block's own share of the result, measured on its own scale
        assert rel_err(got - H64, ref - H64) <= tol, (shape, cfg, rel_err(got - H64, ref - H64))
        assert workspace_is_clean(ws, M, d), (shape, cfg)
        assert torch.equal(g["X"], di.to_torch(t["X"], DEV))          # input untouched
        # in place: bit-identical to the out-of-place result for the ticket reduction
        # (fixed summation order); within tolerance for the atomic one
        h = g["X"].clone()
        dfk.dfk_mlp_block(h, g["w"], eps, g["Wg"], g["Wu"], g["Wd"], h, cfg, ws)
        torch.cuda.synchronize()
        if cfg.reduce == dfk.DFK_REDUCE_TICKET:
            assert torch.equal(h.view(torch.int16), out.view(torch.int16)), (shape, cfg)
        else:
            assert rel_err(y64(h), ref) <= tol, (shape, cfg)
        assert workspace_is_clean(ws, M, d), (shape, cfg)
    # scheduler's choice
    out = torch.empty_like(g["X"])
    dfk.dfk_mlp_block(g["X"], g["w"], eps, g["Wg"], g["Wu"], g["Wd"], out, None, ws)
    assert rel_err(y64(out), ref) <= tol


def test_mlp_block_special_cases():
    """W_down = 0 returns H bit for bit; unit weight and a power-of-two scaling of H leave
    the block's share unchanged (eps = 0); an eps that is not negligible."""
    M, d, ff = 7, 1024, 2816
    t = _block_case(M, d, ff, "bf16", seed=19)
    g = gpu_inputs(t)
    ws = dfk.new_workspace(M, d, ff, DEV)
    out = torch.empty_like(g["X"])
    zero = torch.zeros_like(g["Wd"])
    dfk.dfk_mlp_block(g["X"], g["w"], 1e-5, g["Wg"], g["Wu"], zero, out, None, ws)
    assert torch.equal(out.view(torch.int16), g["X"].view(torch.int16))
    # scaling H by 4 scales nothing but the residual
    dfk.dfk_mlp_block(g["X"], g["w"], 0.0, g["Wg"], g["Wu"], g["Wd"], out, None, ws)
    a = y64(out) - y64(g["X"])
    h4 = (g["X"].float() * 4).to(torch.bfloat16)
    out4 = torch.empty_like(h4)
    dfk.dfk_mlp_block(h4, g["w"], 0.0, g["Wg"], g["Wu"], g["Wd"], out4, None, ws)
    ref4 = oracle.mlp_block(di.to_numpy(h4), t["w"], 0.0, t["Wg"], t["Wu"], t["Wd"])
    assert rel_err(y64(out4), ref4) <= TOL_BF16
    ref1 = oracle.mlp_block(t["X"], t["w"], 0.0, t["Wg"], t["Wu"], t["Wd"])
    np.testing.assert_allclose(ref4 - y64(h4), ref1 - y64(g["X"]), rtol=1e-9, atol=1e-12)   # the oracle agrees it is scale-free
    assert rel_err(y64(out4) - y64(h4), a) <= 3 * TOL_BF16    # two bf16 results, the second rounded on a 4x coarser grid
    # eps three times the mean square (about 1 for these inputs): the normalised input is halved
    eps = 3.0
    dfk.dfk_mlp_block(g["X"], g["w"], eps, g["Wg"], g["Wu"], g["Wd"], out, None, ws)
    ref = oracle.mlp_block(t["X"], t["w"], eps, t["Wg"], t["Wu"], t["Wd"])
    assert rel_err(y64(out), ref) <= TOL_BF16
    assert rel_err(y64(out) - y64(g["X"]), ref - y64(g["X"])) <= TOL_BF16


def test_mlp_block_full_size_sampled_rows():
    """Headline shape, the launch configuration the scheduler picks: sampled tokens against the oracle."""
    d, ff = 4096, 14336
    for M, dtype in ((1, "bf16"), (16, "bf16"), (64, "bf16"), (4, "fp16"), (128, "bf16"), (256, "bf16")):
        g = di.mlp_inputs_torch(M, d, ff, seed=23, dtype=dtype, device=DEV)
        w = di.to_torch(di.tensor(1023, (d,), 1.0, dtype), DEV)
        ws = dfk.new_workspace(M, d, ff, DEV)
        out = torch.empty_like(g["X"])
        print("case full", M, dtype, flush=True)
        dfk.dfk_mlp_block(g["X"], w, 1e-5, g["Wg"], g["Wu"], g["Wd"], out, None, ws)
        torch.cuda.synchronize()
        rows = sorted({0, M - 1, M // 2})
        t = {k: di.to_numpy(v) for k, v in g.items()}
        ref = oracle.mlp_block(t["X"][rows], di.to_numpy(w), 1e-5, t["Wg"], t["Wu"], t["Wd"])
        H = di.as_f64(t["X"][rows])
        got = y64(out)[rows]
        assert_parity(got, ref, dtype, (M, dtype))
        assert rel_err(got - H, ref - H) <= _tol(dtype), (M, dtype)
        assert workspace_is_clean(ws, M, d)


@pytest.mark.parametrize("shape", [(1, 1024, 2816), (16, 512, 4104), (33, 1024, 2816), (64, 2048, 4104), (70, 1024, 2816),
                                   (4, 4096, 14336), (64, 4096, 14336)],
                         ids=lambda s: "M%d_d%d_ff%d" % s)
def test_half_precision_inputs(shape):
    """IEEE half inputs and outputs (the precision the paper evaluates in): every candidate,
    MFMA pair and VALU kernels, against the oracle on the same half bit patterns."""
    M, d, ff = shape
    big = d * ff > 1 << 24
    t = di.mlp_inputs(M, d, ff, seed=13, dtype="fp16") if not big else None
    if big:
        g = di.mlp_inputs_torch(M, d, ff, seed=13, dtype="fp16", device=DEV)
        t = {k: di.to_numpy(v) for k, v in g.items()}
    else:
        g = gpu_inputs(t)
    ref = oracle.swiglu_mlp(t["X"], t["Wg"], t["Wu"], t["Wd"])
    ws = dfk.new_workspace(M, d, ff, DEV)
    n = dfk.dfk_num_candidates(M, d, ff, dfk.DFK_FP16)
    cfgs = [dfk.dfk_get_candidate(M, d, ff, dfk.DFK_FP16, i) for i in range(n)]
    assert any(c.path == dfk.DFK_PATH_VALU for c in cfgs)
    assert any(c.path == dfk.DFK_PATH_MFMA and c.kmajor == 1 for c in cfgs)
    if big:   # the VALU kernels are slow at full size: the MFMA pair and one VALU candidate
        cfgs = [c for c in cfgs if c.path == dfk.DFK_PATH_MFMA][:4] + [c for c in cfgs if c.path == dfk.DFK_PATH_VALU][:1]
    for cfg in cfgs:
        print("case", shape, cfg, flush=True)
        Y, _ = run_ex(g, cfg, ws)
        assert Y.dtype == torch.float16
        assert_parity(y64(Y), ref, "fp16", (shape, cfg))
        assert workspace_is_clean(ws, M, d), (shape, cfg)
    # scheduler's choice through the explicit entry point
    Y = torch.empty_like(g["X"])
    dfk.dfk_swiglu_mlp_ex(g["X"], g["Wg"], g["Wu"], g["Wd"], Y, None, ws)
    assert rel_err(y64(Y), ref) <= TOL_FP16


def test_degenerate_inputs():
    M, d, ff = 4, 512, 1536
    t = di.mlp_inputs(M, d, ff, seed=5)
    g = gpu_inputs(t)
    ws = dfk.new_workspace(M, d, ff, DEV)
    n = dfk.dfk_num_candidates(M, d, ff, dfk.DFK_BF16)
    cfgs = [dfk.dfk_get_candidate(M, d, ff, dfk.DFK_BF16, i) for i in range(n)]
    for cfg in cfgs:
        for zero in ("X", "Wg", "Wu", "Wd"):
            gz = dict(g)
            gz[zero] = torch.zeros_like(g[zero])
            Y, _ = run_ex(gz, cfg, ws)
            assert int(torch.count_nonzero(Y.float()).item()) == 0, (zero, cfg)   # exactly zero
    # extreme gate pre-activations: SiLU -> g for g >> 0, -> 0 for g << 0, no NaN
    big = dict(g)
    big["X"] = g["X"] * 64.0
    big["Wg"] = g["Wg"] * 64.0
    tb = {k: di.to_numpy(v) for k, v in big.items()}
    ref = oracle.swiglu_mlp(tb["X"], tb["Wg"], tb["Wu"], tb["Wd"])
    for cfg in cfgs:
        Y, _ = run_ex(big, cfg, ws)
        assert rel_err(y64(Y), ref) <= TOL_BF16, cfg


@pytest.mark.parametrize("shape,dtype", [((3, 32768, 264), "bf16"), ((64, 32768, 264), "bf16"), ((256, 32768, 72), "bf16"),
                                         ((130, 16384, 264), "bf16"),
                                         ((16, 16384, 1024), "fp16"), ((2, 8, 262144), "bf16"), ((2, 8, 262144), "fp32"),
                                         ((256, 8, 8), "fp32"), ((3, 32768, 264), "fp32")],
                         ids=lambda v: v if isinstance(v, str) else "M%d_d%d_ff%d" % v)
def test_sizes_at_the_limits(shape, dtype):
    """The largest d_model and token count a call accepts (together: four launches of 64 tokens with the
    accumulator area filled to its last byte), a very long and a minimal d_ff, the smallest d_model:
    every candidate the scheduler offers there, against the oracle."""
    M, d, ff = shape
    t = di.mlp_inputs(M, d, ff, seed=77, dtype=dtype)
    ref = oracle.swiglu_mlp(t["X"], t["Wg"], t["Wu"], t["Wd"])
    g = gpu_inputs(t)
    ws = dfk.new_workspace(M, d, ff, DEV)
    n = dfk.dfk_num_candidates(M, d, ff, _dt(dtype))
    assert n > 0
    for i in range(n):
        cfg = dfk.dfk_get_candidate(M, d, ff, _dt(dtype), i)
        assert dfk.dfk_config_valid(cfg, M, d, ff, _dt(dtype))
        print("case", shape, dtype, cfg, flush=True)
        Y, _ = run_ex(g, cfg, ws)
        assert_parity(y64(Y), ref, dtype, (shape, cfg))
        assert workspace_is_clean(ws, M, d), (shape, cfg)
    if dtype != "fp32" and d >= 1024:
        # the block with its neighbours, scheduler's choice, in place
        t["w"] = di.tensor(1077, (d,), 1.0, dtype)
        refb = oracle.mlp_block(t["X"], t["w"], 1e-5, t["Wg"], t["Wu"], t["Wd"])
        h = g["X"].clone()
        print("case block", shape, dtype, flush=True)
        dfk.dfk_mlp_block(h, di.to_torch(t["w"], DEV), 1e-5, g["Wg"], g["Wu"], g["Wd"], h, None, ws)
        torch.cuda.synchronize()
        assert_parity(y64(h), refb, dtype, (shape, "block"))
        assert workspace_is_clean(ws, M, d), shape


def test_repeated_calls_share_a_workspace_and_stay_correct():
    M, d, ff = 4, 1024, 4096
    t = di.mlp_inputs(M, d, ff, seed=9)
    ref = oracle.swiglu_mlp(t["X"], t["Wg"], t["Wu"], t["Wd"])
    g = gpu_inputs(t)
    ws = dfk.new_workspace(M, d, ff, DEV)
    n = dfk.dfk_num_candidates(M, d, ff, dfk.DFK_BF16)
    side = torch.cuda.Stream()
    for i in range(n):
        cfg = dfk.dfk_get_candidate(M, d, ff, dfk.DFK_BF16, i)
        Ys = [torch.empty_like(g["X"]) for _ in range(50)]
        torch.cuda.synchronize()
        with torch.cuda.stream(side):            # a non-default stream, back-to-back launches
            for Y in Ys:
                dfk.dfk_swiglu_mlp_ex(g["X"], g["Wg"], g["Wu"], g["Wd"], Y, cfg, ws)
        torch.cuda.synchronize()
        worst = max(rel_err(y64(Y), ref) for Y in Ys)
        assert worst <= TOL_BF16, (cfg, worst)
        assert workspace_is_clean(ws, M, d)


def test_one_workspace_serves_calls_of_different_token_counts():
    # scratch of one call must never land where a later call with another M expects zeros
    d, ff = 512, 1536
    t = di.mlp_inputs(8, d, ff, seed=17)
    g = gpu_inputs(t)
    ws = dfk.new_workspace(8, d, ff, DEV)
    dfk.dfk_set_workspace(ws)
    try:
        for M in (1, 8, 2, 5, 1, 3):
            ref = oracle.swiglu_mlp(t["X"][:M], t["Wg"], t["Wu"], t["Wd"])
            X = g["X"][:M].contiguous()
            for fn in (dfk.dfk_swiglu_mlp_unfused, dfk.dfk_swiglu_mlp_fused, dfk.dfk_swiglu_mlp):
                Y = torch.full_like(X, float("nan"))
                fn(X, g["Wg"], g["Wu"], g["Wd"], Y)
                torch.cuda.synchronize()
                assert rel_err(y64(Y), ref) <= TOL_BF16, (M, fn.__name__)
                assert workspace_is_clean(ws, M, d)
    finally:
        dfk.dfk_set_workspace(None)


def test_two_host_threads_on_their_own_streams_and_workspaces():
    """Calls from two host threads at once, each on its own stream with its own workspace and its own
    problem (different shapes, kernel families and entry points): the library keeps no state that such
    callers share except the tuning table.  With the counter reduction a result does not depend on what
    else runs, so every call must reproduce, bit for bit, the result the same call gave alone."""
    import threading
    jobs = []
    for k, (M, d, ff, kmajor) in enumerate([(4, 512, 1536, 1), (100, 512, 1000, 2)]):
        t = _block_case(M, d, ff, "bf16", seed=50 + k)
        g = gpu_inputs(t)
        n = dfk.dfk_num_candidates(M, d, ff, dfk.DFK_BF16)
        cfg = next(c for c in (dfk.dfk_get_candidate(M, d, ff, dfk.DFK_BF16, i) for i in range(n))
                   if c.kmajor == kmajor and c.reduce == dfk.DFK_REDUCE_TICKET and c.variant == dfk.DFK_VARIANT_TWO_KERNEL)
        ws = dfk.new_workspace(M, d, ff, DEV)
        alone_y, _ = run_ex(g, cfg, ws)
        alone_b = torch.empty_like(g["X"])
        dfk.dfk_mlp_block(g["X"], g["w"], 1e-5, g["Wg"], g["Wu"], g["Wd"], alone_b, cfg, ws)
        torch.cuda.synchronize()
        assert_parity(y64(alone_y), oracle.swiglu_mlp(t["X"], t["Wg"], t["Wu"], t["Wd"]), "bf16", (M, d, ff))
        assert_parity(y64(alone_b), oracle.mlp_block(t["X"], t["w"], 1e-5, t["Wg"], t["Wu"], t["Wd"]), "bf16", (M, d, ff))
        jobs.append(dict(g=g, cfg=cfg, ws=ws, alone_y=alone_y, alone_b=alone_b, stream=torch.cuda.Stream(), shape=(M, d, ff)))
    torch.cuda.synchronize()
    failures = []
    start = threading.Barrier(len(jobs))

    def worker(j):
        try:
            g, cfg, ws, st = j["g"], j["cfg"], j["ws"], j["stream"]
            ys = [torch.empty_like(g["X"]) for _ in range(60)]
            start.wait()
            for i, y in enumerate(ys):
                if i % 2 == 0:
                    dfk.dfk_swiglu_mlp_ex(g["X"], g["Wg"], g["Wu"], g["Wd"], y, cfg, ws, stream=st)
                else:
                    dfk.dfk_mlp_block(g["X"], g["w"], 1e-5, g["Wg"], g["Wu"], g["Wd"], y, cfg, ws, stream=st)
            st.synchronize()
            for i, y in enumerate(ys):
                want = j["alone_y"] if i % 2 == 0 else j["alone_b"]
                if not torch.equal(y.view(torch.int16), want.view(torch.int16)):
                    failures.append((j["shape"], i))
        except Exception as e:   # reported by the main thread
            failures.append((j["shape"], repr(e)))

    threads = [threading.Thread(target=worker, args=(j,)) for j in jobs]
    for th in threads:
        th.start()
    for th in threads:
        th.join(timeout=120)
    assert not any(th.is_alive() for th in threads)
    assert not failures, failures[:5]
    for j in jobs:
        M, d, _ = j["shape"]
        assert workspace_is_clean(j["ws"], M, d)


def test_split_identity_on_gpu():
    # Appendix A.1 algebra through the GPU path: d_ff shards' outputs sum to the whole.
    M, d, ff = 2, 512, 2048
    t = di.mlp_inputs(M, d, ff, seed=13, dtype="fp32")
    g = gpu_inputs(t)
    ws = dfk.new_workspace(M, d, ff, DEV)
    full, _ = run_ex(g, None, ws)
    tot = torch.zeros_like(full)
    for lo, hi in ((0, 512), (512, 1288), (1288, 2048)):
        gs = {"X": g["X"], "Wg": g["Wg"][lo:hi].contiguous(), "Wu": g["Wu"][lo:hi].contiguous(),
              "Wd": g["Wd"][lo:hi].contiguous()}
        part, _ = run_ex(gs, None, dfk.new_workspace(M, d, hi - lo, DEV))
        tot += part
    assert rel_err(tot.double().cpu().numpy(), full.double().cpu().numpy()) <= 1e-5


def _cfgs(M, d, ff, pred):
    out = []
    for i in range(dfk.dfk_num_candidates(M, d, ff, dfk.DFK_BF16)):
        c = dfk.dfk_get_candidate(M, d, ff, dfk.DFK_BF16, i)
        if pred(c):
            out.append(c)
    return out


@pytest.mark.parametrize("M", [1, 7, 16, 32])
def test_both_reduction_modes_of_the_mfma_path(M):
    d, ff = 1024, 2816
    t = di.mlp_inputs(M, d, ff, seed=23)
    ref = oracle.swiglu_mlp(t["X"], t["Wg"], t["Wu"], t["Wd"])
    g = gpu_inputs(t)
    ws = dfk.new_workspace(M, d, ff, DEV)
    seen = set()
    for c in _cfgs(M, d, ff, lambda c: c.path == dfk.DFK_PATH_MFMA):
        print("case M", M, c, flush=True)
        Y, _ = run_ex(g, c, ws)
        assert rel_err(y64(Y), ref) <= TOL_BF16, (M, c)
        assert workspace_is_clean(ws, M, d)
        seen.add((c.variant, c.reduce))
    for v in (dfk.DFK_VARIANT_FUSED, dfk.DFK_VARIANT_TWO_KERNEL):
        for r in (dfk.DFK_REDUCE_TICKET, dfk.DFK_REDUCE_ATOMIC):
            assert (v, r) in seen


def test_counter_reduction_is_bitwise_reproducible_on_the_valu_path():
    # fixed summation order everywhere on this path: identical bits run after run
    M, d, ff = 4, 1024, 4096
    g = gpu_inputs(di.mlp_inputs(M, d, ff, seed=29))
    ws = dfk.new_workspace(M, d, ff, DEV)
    for c in _cfgs(M, d, ff, lambda c: c.path == dfk.DFK_PATH_VALU)[:4]:
        first, _ = run_ex(g, c, ws)
        for _ in range(20):
            again, _ = run_ex(g, c, ws)
            assert torch.equal(first.view(torch.int16), again.view(torch.int16)), c


def test_counter_reduction_is_bitwise_reproducible_on_the_mfma_path():
    # wavefronts' blocks are added in wavefront order and workgroups' blocks in a fixed order:
    # with the ticket reduction every MFMA form gives identical bits run after run
    for M, d, ff in ((4, 1024, 4096), (40, 1024, 4104)):
        g = gpu_inputs(di.mlp_inputs(M, d, ff, seed=29))
        ws = dfk.new_workspace(M, d, ff, DEV)
        cfgs = _cfgs(M, d, ff, lambda c: c.path == dfk.DFK_PATH_MFMA and c.reduce == dfk.DFK_REDUCE_TICKET)
        forms = {}
        for c in cfgs:   # one of each form
            forms.setdefault((c.variant, c.kmajor, c.k2_rows_by_wave, c.waves), c)
        assert len(forms) >= 4
        for c in forms.values():
            first, _ = run_ex(g, c, ws)
            for _ in range(10):
                again, _ = run_ex(g, c, ws)
                assert torch.equal(first.view(torch.int16), again.view(torch.int16)), c


def test_seeded_random_shapes_and_candidates():
    """A seeded sample of shapes off the beaten path (d_model and d_ff any multiple of 8, token counts on
    and off tile boundaries): the scheduler's default and a few randomly drawn candidates each, bf16 and
    half, against the oracle."""
    import random
    rng = random.Random(815)
    for case in range(14):
        d = 8 * rng.choice([5, 16, 33, 48, 64, 96, 128, 160, 192])
        ff = 8 * rng.choice([2, 9, 33, 70, 125, 257, 352])
        M = rng.choice([1, 3, 15, 16, 17, 31, 33, 48, 63, 64, 65, 97, 129, 255, 256])
        dtype = rng.choice(["bf16", "fp16"])
        t = di.mlp_inputs(M, d, ff, seed=900 + case, dtype=dtype)
        ref = oracle.swiglu_mlp(t["X"], t["Wg"], t["Wu"], t["Wd"])
        g = gpu_inputs(t)
        ws = dfk.new_workspace(M, d, ff, DEV)
        n = dfk.dfk_num_candidates(M, d, ff, _dt(dtype))
        cands = [dfk.dfk_get_candidate(M, d, ff, _dt(dtype), i) for i in range(n)]
        chosen = [None] + rng.sample(cands, min(4, n))
        for cfg in chosen:
            print("case", case, (M, d, ff), dtype, cfg, flush=True)
            Y, _ = run_ex(g, cfg, ws)
            assert_parity(y64(Y), ref, dtype, (case, (M, d, ff), dtype, cfg))
            assert workspace_is_clean(ws, M, d), (case, cfg)


def test_scheduler_tunes_picks_and_reloads(tmp_path):
    """The profile-driven scheduler (Method: a short pre-inference profiling step picks the kernel):
    tune a few token counts on a small shape, check that the picks are valid candidates, that calls
    use them and still match the oracle, that token counts without an entry fall back to the built-in
    default, and that the table survives a save / clear / load."""
    d, ff = 1024, 2816
    Ms = [1, 5, 70]
    dfk.dfk_clear_tuning()
    scratch = torch.empty(dfk.dfk_tune_scratch_bytes(max(Ms), d, ff, dfk.DFK_BF16, 3), dtype=torch.uint8, device=DEV)
    dfk.dfk_tune(Ms, d, ff, dfk.DFK_BF16, scratch, sets=3, iters=3)
    torch.cuda.synchronize()
    picks = {}
    for M in Ms:
        c, tuned = dfk.dfk_get_choice(M, d, ff, dfk.DFK_BF16)
        assert tuned, M
        assert dfk.dfk_config_valid(c, M, d, ff, dfk.DFK_BF16)
        cands = [dfk.dfk_get_candidate(M, d, ff, dfk.DFK_BF16, i).as_dict()
                 for i in range(dfk.dfk_num_candidates(M, d, ff, dfk.DFK_BF16))]
        assert c.as_dict() in cands
        us = dfk.dfk_time_config(c, M, d, ff, dfk.DFK_BF16, scratch, sets=3, iters=3)
        assert 0.5 < us < 5000.0, (M, us)
        picks[M] = c.as_dict()
    assert not dfk.dfk_get_choice(200, d, ff, dfk.DFK_BF16)[1]          # no entry for 200 or its bucket 256
    assert not dfk.dfk_get_choice(1, d, ff, dfk.DFK_FP16)[1]            # another element type
    assert not dfk.dfk_get_choice(1, d, ff + 8, dfk.DFK_BF16)[1]        # another shape
    del scratch
    # calls through the scheduler's choice match the oracle
    ws = dfk.new_workspace(max(Ms), d, ff, DEV)
    dfk.dfk_set_workspace(ws)
    try:
        for M in Ms:
            t = di.mlp_inputs(M, d, ff, seed=37)
            g = gpu_inputs(t)
            Y = torch.empty_like(g["X"])
            dfk.dfk_swiglu_mlp(g["X"], g["Wg"], g["Wu"], g["Wd"], Y)
            torch.cuda.synchronize()
            assert rel_err(y64(Y), oracle.swiglu_mlp(t["X"], t["Wg"], t["Wu"], t["Wd"])) <= TOL_BF16, M
            assert workspace_is_clean(ws, M, d)
    finally:
        dfk.dfk_set_workspace(None)
    path = str(tmp_path / "table.txt")
    dfk.dfk_save_tuning(path)
    dfk.dfk_clear_tuning()
    assert not dfk.dfk_get_choice(5, d, ff, dfk.DFK_BF16)[1]
    dfk.dfk_load_tuning(path)
    for M in Ms:
        c, tuned = dfk.dfk_get_choice(M, d, ff, dfk.DFK_BF16)
        assert tuned and c.as_dict() == picks[M]
    dfk.dfk_clear_tuning()


def test_trace_buffer_records_a_monotone_timeline():
    M, d, ff = 1, 1024, 2816
    g = gpu_inputs(di.mlp_inputs(M, d, ff, seed=31))
    ws = dfk.new_workspace(M, d, ff, DEV)
    c = _cfgs(M, d, ff, lambda c: c.path == dfk.DFK_PATH_MFMA and c.variant == dfk.DFK_VARIANT_FUSED
              and c.reduce == dfk.DFK_REDUCE_TICKET)[0]
    tr = torch.zeros(c.splits * 8, dtype=torch.int64, device=DEV)
    dfk.dfk_set_trace_buffer(tr)
    try:
        run_ex(g, c, ws)
    finally:
        dfk.dfk_set_trace_buffer(None)
    t = tr.cpu().numpy().reshape(-1, 8)
    assert (t[:, 0] > 0).all() and (t[:, 4] >= t[:, 2]).all() and (t[:, 2] >= t[:, 0]).all()
    assert (t[:, 5] >= t[:, 4]).all()
    assert (t[:, 7] > 0).sum() == 1                      # exactly one workgroup wrote Y last
    before = tr.clone()
    run_ex(g, c, ws)                                      # unregistered: nothing is written any more
    assert torch.equal(before, tr)


def test_per_launch_timing_splits_the_two_kernel_variant():
    M, d, ff = 4, 1024, 2816
    scratch = torch.empty(dfk.dfk_tune_scratch_bytes(M, d, ff, dfk.DFK_BF16, 2), dtype=torch.uint8, device=DEV)
    for variant in (dfk.DFK_VARIANT_FUSED, dfk.DFK_VARIANT_TWO_KERNEL):
        c = _cfgs(M, d, ff, lambda c: c.path == dfk.DFK_PATH_MFMA and c.variant == variant)[0]
        whole = dfk.dfk_time_config(c, M, d, ff, dfk.DFK_BF16, scratch, sets=2, iters=10)
        us1, us2 = dfk.dfk_time_kernels(c, M, d, ff, dfk.DFK_BF16, scratch, sets=2, iters=10)
        assert us1 > 0 and whole > 0
        if variant == dfk.DFK_VARIANT_FUSED:
            assert us2 == 0
        else:
            assert us2 > 0
        assert us1 + us2 < 3 * whole + 50      # same order as the whole-call time


def test_read_only_kernel_with_the_gateup_access_pattern():
    """The measurement helper runs on ragged slices and both wavefront counts, leaves the sink alone and
    takes about as long as a streaming read of the same bytes (it reads every byte of both matrices once)."""
    sink = torch.zeros(2, dtype=torch.int32, device=DEV)
    for d, ff, splits in ((1024, 2056, 33), (4096, 14336, 256)):
        w = di.mlp_inputs_torch(1, d, ff, seed=3, device=DEV)
        for waves in (4, 8):
            for _ in range(3):
                dfk.dfk_read_gateup_pattern(w["Wg"], w["Wu"], splits, waves, sink)
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(10):
                dfk.dfk_read_gateup_pattern(w["Wg"], w["Wu"], splits, waves, sink)
            b.record()
            torch.cuda.synchronize()
            us = a.elapsed_time(b) * 100.0
            assert int(sink.abs().sum().item()) == 0
            if d == 4096:     # 234.9 MB: between the 8 TB/s peak and a quarter of it (the weights partly sit in the memory-side cache here)
                assert 234.9e6 / 8e12 * 1e6 * 0.5 < us < 120.0, us


def test_rms_normalize_helper():
    # the weight-free normalisation benchmarks chain layers with (not part of the block)
    for M, d in ((1, 512), (5, 4096), (64, 1000)):
        x = (torch.randn(M, d, device=DEV, generator=torch.Generator(device=DEV).manual_seed(M)) * 3.0).to(torch.bfloat16)
        y = torch.empty_like(x)
        dfk.dfk_rms_normalize(x, y)
        xf = x.double()
        want = xf / xf.pow(2).mean(dim=1, keepdim=True).sqrt()
        assert float((y.double() - want).abs().max()) <= 2.0 ** -7 * float(want.abs().max())


@pytest.mark.parametrize("M", [4, 150])
def test_calls_can_be_captured_in_a_graph_and_replayed(M):
    # the deployment mode of the method: the chosen kernels are captured once and replayed;
    # arrival counters reset themselves, so every replay must equal the eager result
    # (150 tokens: the 256-token pair with its third launch, and several launches of the fused kernel)
    d, ff = 1024, 2816
    t = di.mlp_inputs(M, d, ff, seed=37)
    ref = oracle.swiglu_mlp(t["X"], t["Wg"], t["Wu"], t["Wd"])
    g = gpu_inputs(t)
    ws = dfk.new_workspace(M, d, ff, DEV)
    dfk.dfk_set_workspace(ws)
    try:
        for fn in (dfk.dfk_swiglu_mlp_fused, dfk.dfk_swiglu_mlp_unfused):
            Y = torch.zeros_like(g["X"])
            fn(g["X"], g["Wg"], g["Wu"], g["Wd"], Y)          # eager warm-up (kernel attributes get set here)
            torch.cuda.synchronize()
            eager = Y.clone()
            side = torch.cuda.Stream()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                with torch.cuda.graph(graph, stream=side):
                    fn(g["X"], g["Wg"], g["Wu"], g["Wd"], Y, stream=side)
            for rep in range(5):
                Y.zero_()
                torch.cuda.synchronize()
                graph.replay()
                torch.cuda.synchronize()
                assert rel_err(y64(Y), ref) <= TOL_BF16, (fn.__name__, rep)
                assert rel_err(y64(Y), y64(eager)) <= 1e-2
                # eager work of the program between replays
                fn(g["X"], g["Wg"], g["Wu"], g["Wd"], torch.empty_like(Y))
                torch.cuda.synchronize()
                assert workspace_is_clean(ws, M, d)
        # the block with its neighbours, in place, captured the same way (each replay advances H by one layer)
        w = di.to_torch(di.tensor(1037, (d,), 1.0, "bf16"), DEV)
        h = g["X"].clone()
        dfk.dfk_mlp_block(h, w, 1e-5, g["Wg"], g["Wu"], g["Wd"], h, None, ws)
        torch.cuda.synchronize()
        h.copy_(g["X"])
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                dfk.dfk_mlp_block(h, w, 1e-5, g["Wg"], g["Wu"], g["Wd"], h, None, ws, stream=side)
        cur = di.to_numpy(g["X"])
        for rep in range(3):
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            want = oracle.mlp_block(cur, t_w(w), 1e-5, t["Wg"], t["Wu"], t["Wd"])
            assert rel_err(y64(h), want) <= TOL_BF16, rep
            cur = di.to_numpy(h)                 # teacher forcing: the next layer starts from the GPU's bf16 state
            assert workspace_is_clean(ws, M, d)
    finally:
        dfk.dfk_set_workspace(None)


def t_w(w):
    return di.to_numpy(w)


def test_chained_layers_teacher_forced():
    """Decode sweep shape: distinct 8B-shaped layers chained in stream order, with a
    weight-free RMS normalisation between layers (random SwiGLU layers otherwise
    shrink the activations to zero within a few layers).  Parity is per layer: the
    oracle gets the exact bf16 input the GPU layer got."""
    d, ff, L = 4096, 14336, 6
    for M in (1, 16):
        layers = [di.mlp_inputs_torch(M, d, ff, seed=1000, layer=l, device=DEV) for l in range(L)]
        ws = dfk.new_workspace(M, d, ff, DEV)
        dfk.dfk_set_workspace(ws)
        try:
            X = layers[0]["X"]
            xs, ys = [], []
            for l in range(L):
                Y = torch.empty_like(X)
                dfk.dfk_swiglu_mlp(X, layers[l]["Wg"], layers[l]["Wu"], layers[l]["Wd"], Y)
                xs.append(X)
                ys.append(Y)
                Yf = Y.float()
                X = (Yf / Yf.pow(2).mean(dim=1, keepdim=True).sqrt()).to(torch.bfloat16)
            torch.cuda.synchronize()
            for l in (0, L // 2, L - 1):
                w = layers[l]
                ref = oracle.swiglu_mlp(di.to_numpy(xs[l]), di.to_numpy(w["Wg"]), di.to_numpy(w["Wu"]),
                                        di.to_numpy(w["Wd"]))
                assert np.abs(ref).max() > 1e-2
                assert rel_err(y64(ys[l]), ref) <= TOL_BF16, (M, l)
        finally:
            dfk.dfk_set_workspace(None)


def test_wait_of_the_single_launch_with_both_kernels_is_bounded_and_fails_loudly():
    """The down workgroups of the launch that holds both kernels' workgroups (kmajor = 4) poll a counter of the
    gate/up workgroups; the number of polls is bounded.  With the bound forced to zero from the host every
    workgroup that has to wait gives up at once: the launch must still end, and what such a workgroup contributes
    must be NaN, never a plausible number.  The counters are then out of step with a launch that ran to its end, so
    the workspace is cleared before the next, ordinary call, which must match the oracle again."""
    import os
    M, d, ff = 4, 4096, 14336
    g = di.mlp_inputs_torch(M, d, ff, seed=83, device=DEV)
    host = {k: di.to_numpy(v) for k, v in g.items()}
    ref = oracle.swiglu_mlp(host["X"], host["Wg"], host["Wu"], host["Wd"])
    ws = dfk.new_workspace(M, d, ff, DEV)
    cfg = next(c for c in _cfgs(M, d, ff, lambda c: c.kmajor == 4 and c.reduce == dfk.DFK_REDUCE_TICKET))
    os.environ["DFK_DEBUG_SPIN_LIMIT"] = "0"
    try:
        print("case bounded wait", cfg, flush=True)
        Y = torch.zeros_like(g["X"])
        dfk.dfk_swiglu_mlp_ex(g["X"], g["Wg"], g["Wu"], g["Wd"], Y, cfg, ws)
        torch.cuda.synchronize()                     # the launch ended
    finally:
        del os.environ["DFK_DEBUG_SPIN_LIMIT"]
    got = y64(Y)
    finite = np.isfinite(got)
    cols = finite.all(axis=0)                        # a column is either given up (NaN) or exact
    print("columns given up:", int((~cols).sum()), "of", d, flush=True)
    if cols.any():
        assert rel_err(got[:, cols], ref[:, cols]) <= TOL_BF16
    ws.zero_()
    torch.cuda.synchronize()
    Y, _ = run_ex(g, cfg, ws)
    assert_parity(y64(Y), ref, "bf16", ("after the forced give-up", cfg))
    assert workspace_is_clean(ws, M, d)
