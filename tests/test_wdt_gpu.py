"""GPU parity of the block with the down projection's weights given as W_down_t [d_model, d_ff] (the [out, in]
layout of a linear layer; Background, SwiGLU equations: the same Y = A_2 W_down), through the C ABI against the
fp64 oracle, which takes W_down as the paper writes it.  The device transpose that produces W_down_t is checked
against numpy first."""
import numpy as np
import pytest
import torch

import dfk_inputs as di
import paper_2602_11808_amd as dfk
from oracle import oracle
from tests.helpers import TOL_BF16, assert_parity, rel_err

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
DT = {"bf16": dfk.DFK_BF16, "fp16": dfk.DFK_FP16, "fp32": dfk.DFK_FP32}


def y64(Y):
    return di.as_f64(di.to_numpy(Y))


def transposed(Wd):
    Wd_t = torch.empty((Wd.shape[1], Wd.shape[0]), dtype=Wd.dtype, device=Wd.device)
    dfk.dfk_transpose_w_down(Wd, Wd_t)
    return Wd_t


def cands(M, d, ff, dt):
    return [dfk.dfk_get_candidate_wdt(M, d, ff, dt, i) for i in range(dfk.dfk_num_candidates_wdt(M, d, ff, dt))]


def clean(ws):
    return int(torch.count_nonzero(ws[:4096 + 64 * 32768 * 4]).item()) == 0


@pytest.mark.parametrize("dtype", ["bf16", "fp16", "fp32"])
@pytest.mark.parametrize("shape", [(1000, 520), (14336, 4096), (8, 8), (33, 4104)], ids=lambda s: "%dx%d" % s)
def test_device_transpose_matches_numpy(shape, dtype):
    ff, d = shape
    W = di.tensor(97, (ff, d), 1.0, dtype)
    Wg = di.to_torch(W, DEV)
    got = di.to_numpy(transposed(Wg))
    assert got.shape == (d, ff)
    assert np.array_equal(got.view(np.uint8), np.ascontiguousarray(W.T).view(np.uint8))


@pytest.mark.parametrize("dtype", ["bf16", "fp16", "fp32"])
@pytest.mark.parametrize("shape", [(1, 1024, 2816), (16, 1024, 4224), (17, 2048, 3968), (33, 2048, 4096), (48, 1024, 2816),
                                   (64, 1024, 8192), (100, 1024, 2816), (3, 640, 1152), (40, 2304, 1536), (5, 512, 40960),
                                   (16, 4096, 1024), (1, 8, 8), (3, 264, 1000), (9, 520, 4104), (20, 1024, 2056)],
                         ids=lambda s: "M%d_d%d_ff%d" % s)
def test_every_candidate_of_the_transposed_layout(shape, dtype):
    """One to four token tiles, a token count that needs two launches, d_model with 5 and 18 128-k chunks (uneven k
    split in the gate/up kernel; 144 sixteen-row tiles for the down kernel's slices), a d_ff beyond 512 slices of 64
    rows, d_ff with 8 to 320 chunks for the down kernel's wavefronts; the last four shapes and the fp32 test mode have
    only the plain-FMA pair of this layout (widths that are no multiple of 128, a d_ff that is no multiple of 128);
    every call twice (the workspace must come back clean, the result identical bit for bit: nothing is summed in an
    order that depends on arrival)."""
    M, d, ff = shape
    t = di.mlp_inputs(M, d, ff, seed=41, dtype=dtype)
    ref = oracle.swiglu_mlp(t["X"], t["Wg"], t["Wu"], t["Wd"])
    g = {k: di.to_torch(v, DEV) for k, v in t.items()}
    Wd_t = transposed(g["Wd"])
    ws = dfk.new_workspace(M, d, ff, DEV)
    cfgs = cands(M, d, ff, DT[dtype])
    assert cfgs and all(c.kmajor == 5 and dfk.dfk_config_valid(c, M, d, ff, DT[dtype]) for c in cfgs)
    mfma_ok = dtype != "fp32" and d % 128 == 0 and ff % 128 == 0 and d // 128 >= 4 and ff // 128 >= 4
    assert any(c.path == dfk.DFK_PATH_MFMA for c in cfgs) == mfma_ok
    assert any(c.path == dfk.DFK_PATH_VALU for c in cfgs)
    for cfg in [None] + cfgs:
        print("case", shape, dtype, cfg, flush=True)
        first = None
        for _ in range(2):
            Y = torch.full_like(g["X"], float("nan"))
            dfk.dfk_swiglu_mlp_wdt(g["X"], g["Wg"], g["Wu"], Wd_t, Y, cfg, ws)
            torch.cuda.synchronize()
            assert_parity(y64(Y), ref, dtype, (shape, cfg))
            assert clean(ws), (shape, cfg)
            if first is None:
                first = Y.clone()
            else:
                assert torch.equal(first.view(torch.uint8), Y.view(torch.uint8)), (shape, cfg)


@pytest.mark.parametrize("d,ff", [(4096, 14336), (5120, 27648), (8192, 28672), (8192, 7168)],
                         ids=["llama3_8b", "qwen2.5_32b", "llama3_70b", "tp4_shard_of_70b"])
def test_transposed_layout_full_size(d, ff):
    """The workload's layer shapes at M = 1, 16 and 64 in one launch each: the scheduler's choice for this layout and
    its first and last candidate, sampled tokens against the oracle."""
    g = di.mlp_inputs_torch(64, d, ff, seed=43, device=DEV)
    host = {k: di.to_numpy(v) for k, v in g.items()}
    Wd_t = transposed(g["Wd"])
    ws = dfk.new_workspace(64, d, ff, DEV)
    for M in (1, 16, 64):
        X = g["X"][:M].contiguous()
        rows = list(range(M)) if M <= 16 else [0, 15, 16, 31, 32, 47, 48, 63]
        ref = oracle.swiglu_mlp(host["X"][rows], host["Wg"], host["Wu"], host["Wd"])
        cs = cands(M, d, ff, dfk.DFK_BF16)
        pick, tuned = dfk.dfk_get_choice_wdt(M, d, ff, dfk.DFK_BF16)
        assert not tuned and pick.as_dict() == cs[0].as_dict()
        for cfg in (None, cs[0], cs[-1]):
            print("case full", d, ff, M, cfg, flush=True)
            Y = torch.full_like(X, float("nan"))
            dfk.dfk_swiglu_mlp_wdt(X, g["Wg"], g["Wu"], Wd_t, Y, cfg, ws)
            torch.cuda.synchronize()
            assert bool(torch.isfinite(Y.float()).all())
            assert_parity(y64(Y)[rows], ref, "bf16", (d, ff, M, cfg))
            assert clean(ws)


def test_transposed_layout_in_a_replayed_graph_and_after_tuning():
    """Six chained layers (distinct weights, weight-free normalisation between them) captured once and replayed with
    eager work in between, every layer teacher-forced against the oracle; then dfk_tune on the shape: the choice for
    this layout comes from the table, is one of its candidates, and a call with it still matches."""
    M, d, ff, L = 8, 2048, 4096, 6
    layers = [di.mlp_inputs_torch(M, d, ff, seed=47, layer=l, device=DEV) for l in range(L)]
    wts = [transposed(w["Wd"]) for w in layers]
    host = [{k: di.to_numpy(w[k]) for k in ("Wg", "Wu", "Wd")} for w in layers]
    ws = dfk.new_workspace(M, d, ff, DEV)
    xs = [torch.empty_like(layers[0]["X"]) for _ in range(L + 1)]
    ys = [torch.empty_like(layers[0]["X"]) for _ in range(L)]

    def chain(stream=None):
        for l in range(L):
            dfk.dfk_swiglu_mlp_wdt(xs[l], layers[l]["Wg"], layers[l]["Wu"], wts[l], ys[l], None, ws, stream=stream)
            dfk.dfk_rms_normalize(ys[l], xs[l + 1], stream=stream)

    xs[0].copy_(layers[0]["X"])
    chain()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            chain(stream=side)
    for rep in range(3):
        for t in ys + xs[1:]:
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        print("case graph replay", rep, flush=True)
        graph.replay()
        torch.cuda.synchronize()
        for l in range(L):
            ref = oracle.swiglu_mlp(di.to_numpy(xs[l]), host[l]["Wg"], host[l]["Wu"], host[l]["Wd"])
            assert_parity(y64(ys[l]), ref, "bf16", ("graph", rep, l))
        dfk.dfk_swiglu_mlp_wdt(xs[0], layers[1]["Wg"], layers[1]["Wu"], wts[1], torch.empty_like(xs[0]), None, ws)
        torch.cuda.synchronize()
        assert clean(ws)
    del graph
    scratch = torch.empty(dfk.dfk_tune_scratch_bytes(M, d, ff, dfk.DFK_BF16, 2), dtype=torch.uint8, device=DEV)
    try:
        dfk.dfk_tune([M], d, ff, dfk.DFK_BF16, scratch, sets=2, iters=3)
        pick, tuned = dfk.dfk_get_choice_wdt(M, d, ff, dfk.DFK_BF16)
        assert tuned and pick.kmajor == 5
        assert pick.as_dict() in [c.as_dict() for c in cands(M, d, ff, dfk.DFK_BF16)]
        plain, tuned = dfk.dfk_get_choice(M, d, ff, dfk.DFK_BF16)
        assert tuned and plain.kmajor != 5          # the other layout's entry never becomes the plain choice
        Y = torch.full_like(xs[0], float("nan"))
        dfk.dfk_swiglu_mlp_wdt(layers[0]["X"], layers[0]["Wg"], layers[0]["Wu"], wts[0], Y, None, ws)
        torch.cuda.synchronize()
        ref = oracle.swiglu_mlp(di.to_numpy(layers[0]["X"]), host[0]["Wg"], host[0]["Wu"], host[0]["Wd"])
        assert rel_err(y64(Y), ref) <= TOL_BF16
    finally:
        dfk.dfk_clear_tuning()


@pytest.mark.parametrize("dtype", ["bf16", "fp16"])
@pytest.mark.parametrize("shape", [(1, 1024, 2816), (16, 1024, 4224), (17, 2048, 3968), (64, 1024, 8192), (70, 1024, 2816),
                                   (9, 640, 1152), (4, 4096, 14336)],
                         ids=lambda s: "M%d_d%d_ff%d" % s)
def test_mlp_block_with_norm_and_residual_transposed_layout(shape, dtype):
    """H + MLP(RMSNorm(H)) with W_down_t, against the oracle's composition: every candidate of the layout, out of
    place and in place (bit-identical: nothing depends on arrival order), the input untouched, and a configuration
    of the other layout refused."""
    M, d, ff = shape
    eps = 1e-5
    t = di.mlp_inputs(M, d, ff, seed=53, dtype=dtype)
    t["w"] = di.tensor(1053, (d,), 1.0, dtype)
    ref = oracle.mlp_block(t["X"], t["w"], eps, t["Wg"], t["Wu"], t["Wd"])
    H64 = di.as_f64(t["X"])
    g = {k: di.to_torch(v, DEV) for k, v in t.items()}
    Wd_t = transposed(g["Wd"])
    ws = dfk.new_workspace(M, d, ff, DEV)
    tol = {"bf16": TOL_BF16, "fp16": 2e-3}[dtype]
    other = dfk.dfk_get_candidate(M, d, ff, DT[dtype], 0)
    with pytest.raises(dfk.DfkError) as ei:
        dfk.dfk_mlp_block_wdt(g["X"], g["w"], eps, g["Wg"], g["Wu"], Wd_t, torch.empty_like(g["X"]), other, ws)
    assert ei.value.status == dfk.DFK_ERR_INVALID_ARG
    cfgs = [c for c in cands(M, d, ff, DT[dtype]) if c.path == dfk.DFK_PATH_MFMA]   # the plain-FMA pair does not carry the block
    valu = next(c for c in cands(M, d, ff, DT[dtype]) if c.path == dfk.DFK_PATH_VALU)
    with pytest.raises(dfk.DfkError) as ei:
        dfk.dfk_mlp_block_wdt(g["X"], g["w"], eps, g["Wg"], g["Wu"], Wd_t, torch.empty_like(g["X"]), valu, ws)
    assert ei.value.status == dfk.DFK_ERR_UNSUPPORTED_SHAPE
    if d * ff > 1 << 24:
        cfgs = cfgs[:2]
    for cfg in [None] + cfgs:
        print("case block", shape, dtype, cfg, flush=True)
        out = torch.full_like(g["X"], float("nan"))
        dfk.dfk_mlp_block_wdt(g["X"], g["w"], eps, g["Wg"], g["Wu"], Wd_t, out, cfg, ws)
        torch.cuda.synchronize()
        got = y64(out)
        assert_parity(got, ref, dtype, (shape, cfg))
        assert rel_err(got - H64, ref - H64) <= tol, (shape, cfg, rel_err(got - H64, ref - H64))
        assert clean(ws)
        assert torch.equal(g["X"], di.to_torch(t["X"], DEV))
        h = g["X"].clone()
        dfk.dfk_mlp_block_wdt(h, g["w"], eps, g["Wg"], g["Wu"], Wd_t, h, cfg, ws)
        torch.cuda.synchronize()
        assert torch.equal(h.view(torch.int16), out.view(torch.int16)), (shape, cfg)
        assert clean(ws)


def test_a_thousand_launches_in_the_transposed_layout_give_identical_bits():
    """No workgroup of this layout's down kernel sums another's partial result, so at the headline shape 1000 launches
    in a row must reproduce the first result bit for bit, whatever order the workgroups run in; stops at the first
    mismatch."""
    d, ff = 4096, 14336
    for M in (4, 16):
        g = di.mlp_inputs_torch(M, d, ff, seed=59, device=DEV)
        Wd_t = transposed(g["Wd"])
        ws = dfk.new_workspace(M, d, ff, DEV)
        first = torch.empty_like(g["X"])
        dfk.dfk_swiglu_mlp_wdt(g["X"], g["Wg"], g["Wu"], Wd_t, first, None, ws)
        Y = torch.empty_like(first)
        print("case 1000 launches M", M, flush=True)
        for i in range(1000):
            dfk.dfk_swiglu_mlp_wdt(g["X"], g["Wg"], g["Wu"], Wd_t, Y, None, ws)
            if i % 10 == 9 or i < 10:
                assert torch.equal(first.view(torch.int16), Y.view(torch.int16)), (M, i)
                Y.fill_(float("nan"))
        torch.cuda.synchronize()
