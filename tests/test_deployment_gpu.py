"""GPU parity in the paper's deployment mode and on its per-GPU workload (through the C ABI, against
the fp64 oracle): a whole 32-layer decode pass captured once in a HIP graph and replayed
(Experiment Setup: graphs enabled; Method: no dispatch cost at inference), the per-GPU shard of the
70B layer under four-way tensor parallelism in both 16-bit types (Experiment Setup; Appendix A.1),
long runs of the deterministic reduction, and the d_ff permutation invariance of the block."""
import numpy as np
import pytest
import torch

import dfk_inputs as di
import paper_2602_11808_amd as dfk
from oracle import oracle
from tests.helpers import TOL_BF16, TOL_FP16, TOL_FP32, assert_parity, rel_err

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
D8B, FF8B = 4096, 14336


def y64(Y):
    return di.as_f64(di.to_numpy(Y))


def _forms(M, d, ff, dt, pred=lambda c: True):
    """One candidate of each kernel form (variant, path, family, reduction)."""
    forms = {}
    for i in range(dfk.dfk_num_candidates(M, d, ff, dt)):
        c = dfk.dfk_get_candidate(M, d, ff, dt, i)
        if pred(c):
            forms.setdefault((c.variant, c.path, c.kmajor, c.k2_rows_by_wave, c.reduce), c)
    return list(forms.values())


def test_decode_pass_of_32_layers_captured_once_and_replayed():
    """32 chained 8B-shaped layers with distinct weights (11.3 GB, far beyond any cache), a weight-free RMS
    normalisation between layers, the whole pass captured once and replayed three times with eager work in
    between.  After every replay sampled layers are checked against the oracle, teacher-forced: the oracle
    gets the exact bf16 input that the GPU layer read in that replay."""
    L = 32
    layers = [di.mlp_inputs_torch(1, D8B, FF8B, seed=1000, layer=l, device=DEV) for l in range(L)]
    sampled = (0, 13, L - 1)
    host_w = {l: {k: di.to_numpy(layers[l][k]) for k in ("Wg", "Wu", "Wd")} for l in sampled}
    ws = dfk.new_workspace(256, D8B, FF8B, DEV)
    dfk.dfk_set_workspace(ws)
    try:
        for M in (1, 16, 256):
            X0 = di.mlp_inputs_torch(M, D8B, FF8B, seed=7, layer=0, device=DEV)["X"]
            xs = [torch.empty_like(X0) for _ in range(L + 1)]
            ys = [torch.empty_like(X0) for _ in range(L)]

            def chain(stream=None):
                for l in range(L):
                    w = layers[l]
                    dfk.dfk_swiglu_mlp(xs[l], w["Wg"], w["Wu"], w["Wd"], ys[l], stream=stream)
                    dfk.dfk_rms_normalize(ys[l], xs[l + 1], stream=stream)

            xs[0].copy_(X0)
            chain()                                   # eager warm-up: kernel attributes get set outside the capture
            torch.cuda.synchronize()
            side = torch.cuda.Stream()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                with torch.cuda.graph(graph, stream=side):
                    chain(stream=side)
            rows = list(range(M)) if M <= 16 else [0, 15, 16, 77, M - 1]
            for rep in range(3):
                for t in ys + xs[1:]:
                    t.fill_(float("nan"))
                torch.cuda.synchronize()
                print("case decode32 M", M, "replay", rep, flush=True)
                graph.replay()
                torch.cuda.synchronize()
                assert bool(torch.isfinite(xs[L].float()).all()), (M, rep)
                for l in sampled:
                    ref = oracle.swiglu_mlp(di.to_numpy(xs[l])[rows], host_w[l]["Wg"], host_w[l]["Wu"], host_w[l]["Wd"])
                    assert np.abs(ref).max() > 1e-2
                    assert_parity(y64(ys[l])[rows], ref, "bf16", ("decode32", M, rep, l))
                # eager work of the program between replays, on the same workspace
                dfk.dfk_swiglu_mlp(xs[0], layers[1]["Wg"], layers[1]["Wu"], layers[1]["Wd"], torch.empty_like(X0))
                torch.cuda.synchronize()
                assert int(torch.count_nonzero(ws[:4096 + 64 * 32768 * 4]).item()) == 0
            del graph
    finally:
        dfk.dfk_set_workspace(None)


@pytest.mark.parametrize("dtype", ["bf16", "fp16"])
def test_tensor_parallel_shard_shape_of_the_70b_layer(dtype):
    """d_model = 8192, d_ff = 28672 / 4 = 7168: what one GPU computes of the 70B layer under four-way tensor
    parallelism (Appendix A.1: W_gate, W_up split by d_ff columns, W_down by d_ff rows), in the precision of
    the paper's experiments (half) and in bf16; the scheduler's choice and one candidate of every MFMA form."""
    d, ff = 8192, 7168
    dt = {"bf16": dfk.DFK_BF16, "fp16": dfk.DFK_FP16}[dtype]
    g = di.mlp_inputs_torch(64, d, ff, seed=61, dtype=dtype, device=DEV)
    host = {k: di.to_numpy(v) for k, v in g.items()}
    ws = dfk.new_workspace(64, d, ff, DEV)
    for M in (1, 16, 64):
        X = g["X"][:M].contiguous()
        rows = list(range(M)) if M <= 16 else [0, 1, 15, 16, 31, 32, 47, 48, 62, 63]
        ref = oracle.swiglu_mlp(host["X"][rows], host["Wg"], host["Wu"], host["Wd"])
        cfgs = [None] + _forms(M, d, ff, dt, lambda c: c.path == dfk.DFK_PATH_MFMA)
        assert len(cfgs) >= 3
        for cfg in cfgs:
            print("case tp4 shard", dtype, M, cfg, flush=True)
            Y = torch.full_like(X, float("nan"))
            dfk.dfk_swiglu_mlp_ex(X, g["Wg"], g["Wu"], g["Wd"], Y, cfg, ws)
            torch.cuda.synchronize()
            assert_parity(y64(Y)[rows], ref, dtype, ("tp4", dtype, M, cfg))
            assert int(torch.count_nonzero(ws[:4096 + 64 * 32768 * 4]).item()) == 0


def test_a_thousand_launches_of_every_deterministic_form_give_identical_bits():
    """The counter reduction adds the partial sums in a fixed order, whatever order the workgroups (on eight
    XCDs with an L2 each) arrive in: at the headline shape 1000 launches in a row of every MFMA form with that
    reduction must reproduce the first result bit for bit; stops at the first mismatch."""
    for M in (4, 16):
        g = di.mlp_inputs_torch(M, D8B, FF8B, seed=67, device=DEV)
        ws = dfk.new_workspace(M, D8B, FF8B, DEV)
        forms = _forms(M, D8B, FF8B, dfk.DFK_BF16,
                       lambda c: c.path == dfk.DFK_PATH_MFMA and c.reduce == dfk.DFK_REDUCE_TICKET)
        assert len(forms) >= 3
        for cfg in forms:
            print("case 1000 launches M", M, cfg, flush=True)
            first = torch.empty_like(g["X"])
            dfk.dfk_swiglu_mlp_ex(g["X"], g["Wg"], g["Wu"], g["Wd"], first, cfg, ws)
            Y = torch.empty_like(first)
            for i in range(1000):
                dfk.dfk_swiglu_mlp_ex(g["X"], g["Wg"], g["Wu"], g["Wd"], Y, cfg, ws)
                if i % 10 == 9 or i < 10:          # the comparison synchronises; most launches run back to back
                    assert torch.equal(first.view(torch.int16), Y.view(torch.int16)), (M, cfg, i)
                    Y.fill_(float("nan"))
            torch.cuda.synchronize()


@pytest.mark.parametrize("dtype,tol", [("fp32", TOL_FP32), ("bf16", TOL_BF16), ("fp16", TOL_FP16)])
def test_permuting_d_ff_leaves_the_result_unchanged_on_the_gpu(dtype, tol):
    """Permuting the d_ff index of W_gate, W_up and W_down together changes which slice every row lands in and
    the order of every sum, and nothing else: each candidate form must return the same Y within the stated
    tolerance (fp32 test mode: 1e-5), and both must match the oracle."""
    M, d, ff = 5, 1024, 2816
    dt = {"bf16": dfk.DFK_BF16, "fp16": dfk.DFK_FP16, "fp32": dfk.DFK_FP32}[dtype]
    t = di.mlp_inputs(M, d, ff, seed=71, dtype=dtype)
    perm = np.random.default_rng(71).permutation(ff)
    tp = dict(t, Wg=np.ascontiguousarray(t["Wg"][perm]), Wu=np.ascontiguousarray(t["Wu"][perm]),
              Wd=np.ascontiguousarray(t["Wd"][perm]))
    ref = oracle.swiglu_mlp(t["X"], t["Wg"], t["Wu"], t["Wd"])
    g = {k: di.to_torch(v, DEV) for k, v in t.items()}
    gp = {k: di.to_torch(v, DEV) for k, v in tp.items()}
    ws = dfk.new_workspace(M, d, ff, DEV)
    for cfg in [None] + _forms(M, d, ff, dt):
        print("case permutation", dtype, cfg, flush=True)
        Y, Yp = torch.full_like(g["X"], float("nan")), torch.full_like(g["X"], float("nan"))
        dfk.dfk_swiglu_mlp_ex(g["X"], g["Wg"], g["Wu"], g["Wd"], Y, cfg, ws)
        dfk.dfk_swiglu_mlp_ex(gp["X"], gp["Wg"], gp["Wu"], gp["Wd"], Yp, cfg, ws)
        torch.cuda.synchronize()
        assert_parity(y64(Y), ref, dtype, ("perm", dtype, cfg))
        assert_parity(y64(Yp), ref, dtype, ("perm", dtype, cfg, "permuted"))
        assert rel_err(y64(Yp), y64(Y)) <= tol, (dtype, cfg)
