"""The entry point that allocates nothing (dfk_swiglu_mlp_static: scratch in an array of the library's
own code object) against dfk_swiglu_mlp_ex on a caller's workspace, through the C ABI: same
configuration, same inputs, two calls in a row of which the second is smaller.  With the counter
reduction the summation order is fixed, so the two entry points must agree bit for bit; with the
atomic reduction within the stated tolerance.  Both are also held against the oracle."""
import pytest
import torch

import dfk_inputs as di
import paper_2602_11808_amd as dfk
from oracle import oracle
from tests.helpers import assert_parity, rel_err, TOL_BF16, TOL_FP16, TOL_FP32

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
_DT = {"bf16": dfk.DFK_BF16, "fp32": dfk.DFK_FP32, "fp16": dfk.DFK_FP16}
_TOL = {"bf16": TOL_BF16, "fp32": TOL_FP32, "fp16": TOL_FP16}


def _y64(Y):
    return di.as_f64(di.to_numpy(Y))


def _one_of_each_form(M, d, ff, dtype):
    forms = {}
    for i in range(dfk.dfk_num_candidates(M, d, ff, _DT[dtype])):
        c = dfk.dfk_get_candidate(M, d, ff, _DT[dtype], i)
        forms.setdefault((c.variant, c.path, c.kmajor, c.k2_rows_by_wave, c.reduce), c)
    return list(forms.values())


@pytest.mark.parametrize("dtype,first,second", [
    ("bf16", (16, 1024, 2816), (3, 512, 1000)),
    ("fp16", (40, 1024, 4104), (1, 1024, 4104)),
    ("fp32", (5, 520, 4104), (2, 264, 1000)),
    ("bf16", (130, 512, 1536), (64, 512, 1536)),
], ids=["bf16", "fp16", "fp32", "bf16_many_tokens"])
def test_static_scratch_entry_point_matches_the_workspace_entry_point(dtype, first, second):
    cases = []
    for shape in (first, second):
        M, d, ff = shape
        t = di.mlp_inputs(M, d, ff, seed=41, dtype=dtype)
        cases.append((shape, t, {k: di.to_torch(v, DEV) for k, v in t.items()},
                      oracle.swiglu_mlp(t["X"], t["Wg"], t["Wu"], t["Wd"]), dfk.new_workspace(M, d, ff, DEV)))
    cfgs_first = [None] + _one_of_each_form(*first, dtype)
    for cfg1 in cfgs_first:
        # two calls in a row on the library's array, the second with the smaller input
        outs = []
        for k, (shape, t, g, ref, ws) in enumerate(cases):
            M, d, ff = shape
            cfg = cfg1 if k == 0 else (None if cfg1 is None else _match(cfg1, shape, dtype))
            print("case", dtype, shape, cfg, flush=True)
            Ys = torch.full_like(g["X"], float("nan"))
            dfk.dfk_swiglu_mlp_static(g["X"], g["Wg"], g["Wu"], g["Wd"], Ys, cfg)
            outs.append((shape, g, ref, ws, cfg, Ys))
        torch.cuda.synchronize()
        for shape, g, ref, ws, cfg, Ys in outs:
            Ye = torch.full_like(g["X"], float("nan"))
            dfk.dfk_swiglu_mlp_ex(g["X"], g["Wg"], g["Wu"], g["Wd"], Ye, cfg, ws)
            torch.cuda.synchronize()
            assert_parity(_y64(Ys), ref, dtype, (shape, cfg, "static"))
            assert_parity(_y64(Ye), ref, dtype, (shape, cfg, "ex"))
            used = cfg if cfg is not None else dfk.dfk_get_choice(*shape, _DT[dtype])[0]
            if used.reduce == dfk.DFK_REDUCE_TICKET:
                assert torch.equal(Ys.view(torch.uint8), Ye.view(torch.uint8)), (shape, cfg)
            else:
                assert rel_err(_y64(Ys), _y64(Ye)) <= _TOL[dtype], (shape, cfg)


def _match(cfg, shape, dtype):
    """A candidate of the second shape of the same form as cfg (else the scheduler's choice)."""
    M, d, ff = shape
    for c in _one_of_each_form(M, d, ff, dtype):
        if (c.variant, c.path, c.kmajor, c.k2_rows_by_wave, c.reduce) == \
                (cfg.variant, cfg.path, cfg.kmajor, cfg.k2_rows_by_wave, cfg.reduce):
            return c
    return None


def test_static_scratch_at_the_headline_shape_and_its_limits():
    d, ff = 4096, 14336
    g = di.mlp_inputs_torch(16, d, ff, seed=43, device=DEV)
    host = {k: di.to_numpy(v) for k, v in g.items()}
    ws = dfk.new_workspace(16, d, ff, DEV)
    for M in (16, 1):       # the second call smaller than the first
        X = g["X"][:M].contiguous()
        ref = oracle.swiglu_mlp(host["X"][:M], host["Wg"], host["Wu"], host["Wd"])
        Ys, Ye = torch.full_like(X, float("nan")), torch.full_like(X, float("nan"))
        print("case headline", M, flush=True)
        dfk.dfk_swiglu_mlp_static(X, g["Wg"], g["Wu"], g["Wd"], Ys)
        dfk.dfk_swiglu_mlp_ex(X, g["Wg"], g["Wu"], g["Wd"], Ye, None, ws)
        torch.cuda.synchronize()
        assert_parity(_y64(Ys), ref, "bf16", ("headline", M, "static"))
        assert rel_err(_y64(Ys), _y64(Ye)) <= TOL_BF16
    # beyond the array: refused before any launch, and the output is not touched
    M, d, ff = 256, 512, 16392                      # A_2 of 256 x 16392 fp32 exceeds its 16 MiB share
    X = torch.zeros(M, d, dtype=torch.bfloat16, device=DEV)
    W = torch.zeros(ff, d, dtype=torch.bfloat16, device=DEV)
    Y = torch.full_like(X, 7.0)
    with pytest.raises(dfk.DfkError) as ei:
        dfk.dfk_swiglu_mlp_static(X, W, W, W, Y)
    assert ei.value.status == dfk.DFK_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((Y == 7.0).all())
