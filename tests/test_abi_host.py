"""Host-side checks that need no GPU: the library loads, exports every symbol
the header declares, validates arguments before touching HIP, and keeps the
scheduler table (set / get / save / load / clear)."""
import ctypes
import os
import re
import subprocess

import pytest

import paper_2602_11808_amd as dfk

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
D, FF = 4096, 14336
A = 0x10000000          # fake, well-aligned, non-overlapping "device" addresses
X, WG, WU, WD, Y, WS = A, 2 * A, 3 * A, 4 * A, 5 * A, 6 * A


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "dfk.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(dfk_[a-z_0-9]+)\s*\(", header))
    assert len(declared) >= 20
    l = ctypes.CDLL(dfk.LIB_PATH)
    for name in declared:
        assert hasattr(l, name), f"{name} declared in dfk.h but not exported"
    bound = {n for n, _, _ in dfk.binding.SIGNATURES}
    assert declared == bound, declared ^ bound
    for name in declared:
        if name.startswith("dfk_") and name not in ("dfk_config_t",):
            assert hasattr(dfk, name), f"binding lacks {name}"
    assert "gfx950" in dfk.dfk_version()


def test_header_is_plain_c_and_a_c_program_can_call_the_library(tmp_path):
    """The boundary is a C ABI: the header compiles as strict C99 and as C++, a C program links
    against the library and calls its host-only entry points, and the configuration struct has
    the layout the Python binding assumes."""
    inc = os.path.join(ROOT, "include")
    src = tmp_path / "use_dfk.c"
    src.write_text(r"""
#include <stddef.h>
#include <stdio.h>
#include "dfk.h"
int main(void) {
    dfk_config_t c;
    int n = dfk_num_candidates(4, 4096, 14336, DFK_BF16);
    if (n < 1 || dfk_get_candidate(4, 4096, 14336, DFK_BF16, 0, &c) != DFK_OK) return 2;
    if (!dfk_config_valid(&c, 4, 4096, 14336, DFK_BF16)) return 3;
    if (dfk_check_args((const void*)0x10000000, (const void*)0x20000000, (const void*)0x30000000,
                       (const void*)0x40000000, (const void*)0x50000000, 4, 4096, 14336, DFK_BF16, &c, NULL, 0) != DFK_OK) return 4;
    if (dfk_check_args(NULL, NULL, NULL, NULL, NULL, 4, 4096, 14336, DFK_BF16, NULL, NULL, 0) == DFK_OK) return 5;
    printf("%d %d %d %d %d %s\n", (int)sizeof(dfk_config_t), (int)offsetof(dfk_config_t, variant),
           (int)offsetof(dfk_config_t, k2_splits), (int)offsetof(dfk_config_t, kmajor), n, dfk_version());
    return 0;
}
""")
    subprocess.check_call(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", inc, "-fsyntax-only", str(src)])
    cxx = tmp_path / "use_dfk.cpp"
    cxx.write_text('#include "dfk.h"\nint main() { return dfk_status_string(DFK_OK) ? 0 : 1; }\n')
    subprocess.check_call(["g++", "-std=c++11", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", inc, "-fsyntax-only", str(cxx)])
    exe = tmp_path / "use_dfk"
    libdir = os.path.dirname(dfk.LIB_PATH)
    subprocess.check_call(["gcc", "-std=c99", "-I", inc, "-o", str(exe), str(src), "-L", libdir, "-ldfk",
                           "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib"])
    out = subprocess.run([str(exe)], stdout=subprocess.PIPE, text=True, timeout=120)
    assert out.returncode == 0, out.returncode
    size, o_variant, o_k2s, o_kmajor, n, version = out.stdout.split(None, 5)
    assert int(size) == ctypes.sizeof(dfk.dfk_config_t)
    assert int(o_variant) == dfk.dfk_config_t.variant.offset
    assert int(o_k2s) == dfk.dfk_config_t.k2_splits.offset
    assert int(o_kmajor) == dfk.dfk_config_t.kmajor.offset
    assert int(n) == dfk.dfk_num_candidates(4, 4096, 14336, dfk.DFK_BF16)
    assert "gfx950" in version


def chk(**kw):
    a = dict(X=X, W_gate=WG, W_up=WU, W_down=WD, Y=Y, M=1, d_model=D, d_ff=FF)
    a.update(kw)
    return dfk.dfk_check_args(**a)


def test_valid_arguments_pass():
    assert chk() == dfk.DFK_OK
    assert chk(M=256) == dfk.DFK_OK
    assert chk(dtype=dfk.DFK_FP32) == dfk.DFK_OK
    n = dfk.dfk_workspace_bytes(16, D, FF)
    assert chk(M=16, workspace=WS, workspace_bytes=n) == dfk.DFK_OK


def test_invalid_arguments():
    for name in ("X", "W_gate", "W_up", "W_down", "Y"):
        assert chk(**{name: 0}) == dfk.DFK_ERR_INVALID_ARG
    assert chk(M=0) == dfk.DFK_ERR_INVALID_ARG
    assert chk(M=-3) == dfk.DFK_ERR_INVALID_ARG
    assert chk(d_model=0) == dfk.DFK_ERR_INVALID_ARG
    assert chk(d_ff=-8) == dfk.DFK_ERR_INVALID_ARG
    assert chk(dtype=7) == dfk.DFK_ERR_INVALID_ARG


def test_unsupported_shapes():
    assert chk(d_model=4100) == dfk.DFK_ERR_UNSUPPORTED_SHAPE
    assert chk(d_ff=14340) == dfk.DFK_ERR_UNSUPPORTED_SHAPE
    assert chk(M=dfk.DFK_MAX_M + 1) == dfk.DFK_ERR_UNSUPPORTED_SHAPE


def test_alignment_and_alias():
    assert chk(X=X + 8) == dfk.DFK_ERR_ALIGNMENT
    assert chk(W_down=WD + 2) == dfk.DFK_ERR_ALIGNMENT
    assert chk(Y=X) == dfk.DFK_ERR_ALIAS
    assert chk(Y=WG + 4096) == dfk.DFK_ERR_ALIAS              # inside W_gate
    assert chk(M=4, Y=X + 2 * D * 2) == dfk.DFK_ERR_ALIAS      # overlaps later rows of X
    assert chk(M=1, Y=X + 1 * D * 2) == dfk.DFK_OK             # just past a 1-row X


def test_workspace_checks():
    n = dfk.dfk_workspace_bytes(8, D, FF)
    assert n >= 4096 + 64 * 32768 * 4 + 256 * 8 * D * 4 + 8 * FF * 4
    assert dfk.dfk_workspace_bytes(0, D, FF) == 0 and dfk.dfk_workspace_bytes(1, 0, FF) == 0
    assert chk(M=8, workspace=0, workspace_bytes=n) == dfk.DFK_ERR_WORKSPACE
    assert chk(M=8, workspace=WS, workspace_bytes=n - 1) == dfk.DFK_ERR_WORKSPACE
    assert chk(M=8, workspace=WS + 16, workspace_bytes=n) == dfk.DFK_ERR_ALIGNMENT
    assert chk(M=8, workspace=Y, workspace_bytes=n) == dfk.DFK_ERR_ALIAS
    # the non-_ex entry points refuse to run without a registered workspace (no HIP call made)
    dfk.dfk_set_workspace(None)
    st = dfk.lib().dfk_swiglu_mlp(X, WG, WU, WD, Y, 1, D, FF, None)
    assert st == dfk.DFK_ERR_WORKSPACE
    assert dfk.lib().dfk_swiglu_mlp_fused(X, WG, WU, WD, Y, 0, D, FF, None) == dfk.DFK_ERR_INVALID_ARG
    assert dfk.lib().dfk_swiglu_mlp_unfused(0, WG, WU, WD, Y, 1, D, FF, None) == dfk.DFK_ERR_INVALID_ARG


def test_config_validation():
    n = dfk.dfk_num_candidates(4, D, FF, dfk.DFK_BF16)
    assert n > 0
    seen_variants = set()
    for i in range(n):
        c = dfk.dfk_get_candidate(4, D, FF, dfk.DFK_BF16, i)
        assert dfk.dfk_config_valid(c, 4, D, FF, dfk.DFK_BF16)
        assert chk(M=4, cfg=c) == dfk.DFK_OK
        seen_variants.add(c.variant)
    assert seen_variants == {dfk.DFK_VARIANT_FUSED, dfk.DFK_VARIANT_TWO_KERNEL}
    with pytest.raises(dfk.DfkError):
        dfk.dfk_get_candidate(4, D, FF, dfk.DFK_BF16, n)
    bad = dfk.dfk_get_candidate(4, D, FF, dfk.DFK_BF16, 0)
    bad.splits = 0
    assert not dfk.dfk_config_valid(bad, 4, D, FF, dfk.DFK_BF16)
    assert chk(M=4, cfg=bad) == dfk.DFK_ERR_UNSUPPORTED_SHAPE
    bad.splits, bad.variant = 256, 9
    assert chk(M=4, cfg=bad) == dfk.DFK_ERR_INVALID_ARG
    # fp32 test mode never gets the bf16 MFMA path
    for i in range(dfk.dfk_num_candidates(4, D, FF, dfk.DFK_FP32)):
        assert dfk.dfk_get_candidate(4, D, FF, dfk.DFK_FP32, i).path == dfk.DFK_PATH_VALU
    assert dfk.dfk_num_candidates(4, 4100, FF, dfk.DFK_BF16) == 0


def test_kernel_families_by_token_count():
    """The 64-token pair is offered at every token count, the 256-token pair beyond 64 tokens only; the
    untuned default follows (one token: the single launch with A_2 in LDS; up to 64: the single launch of both
    kernels' workgroups; beyond: the 256-token pair; two-kernel variant asked for: the pairs); the limits of the
    256-token pair are enforced on the host."""
    import copy
    for dt in (dfk.DFK_BF16, dfk.DFK_FP16):
        for M, want2 in ((1, False), (64, False), (65, True), (128, True), (256, True)):
            cands = [dfk.dfk_get_candidate(M, D, FF, dt, i) for i in range(dfk.dfk_num_candidates(M, D, FF, dt))]
            assert any(c.kmajor == 1 for c in cands)
            assert any(c.kmajor == 2 for c in cands) == want2
            for c in cands:
                assert dfk.dfk_config_valid(c, M, D, FF, dt), (M, c)
            pick, tuned = dfk.dfk_get_choice(M, D, FF, dt)
            assert not tuned
            assert (pick.variant, pick.kmajor) == ((dfk.DFK_VARIANT_TWO_KERNEL, 2) if want2 else
                                                   (dfk.DFK_VARIANT_FUSED, 1 if M == 1 else 4))
            assert any(c.kmajor == 4 and c.variant == dfk.DFK_VARIANT_FUSED for c in cands)
    assert dfk.dfk_num_candidates(128, D, FF, dfk.DFK_FP32) > 0          # fp32 test mode: VALU kernels only
    assert all(dfk.dfk_get_candidate(128, D, FF, dfk.DFK_FP32, i).path == dfk.DFK_PATH_VALU
               for i in range(dfk.dfk_num_candidates(128, D, FF, dfk.DFK_FP32)))
    big = next(c for c in (dfk.dfk_get_candidate(256, D, FF, dfk.DFK_BF16, i)
                         for i in range(dfk.dfk_num_candidates(256, D, FF, dfk.DFK_BF16))) if c.kmajor == 2)
    for field, bad in (("waves", 2), ("waves", 16), ("depth", 2), ("depth", 5), ("k2_col_blocks", 16), ("splits", 128),
                       ("a2_dtype", dfk.DFK_FP32), ("k2_rows_by_wave", 1), ("variant", dfk.DFK_VARIANT_FUSED)):
        c = copy.copy(big)
        setattr(c, field, bad)
        assert not dfk.dfk_config_valid(c, 256, D, FF, dfk.DFK_BF16), (field, bad)
    # the fp32 accumulator of one launch holds 8 MiB: 256 tokens x d_model 16384 do not fit it, which
    # rules out the atomic mode there; the counter mode keeps its partial blocks elsewhere and runs
    wide = copy.copy(big)
    wide.k2_col_blocks = 16384 // 128
    wide.k2_splits = 2
    wide.reduce = dfk.DFK_REDUCE_ATOMIC
    assert not dfk.dfk_config_valid(wide, 256, 16384, FF, dfk.DFK_BF16)
    wide.reduce = dfk.DFK_REDUCE_TICKET
    assert dfk.dfk_config_valid(wide, 256, 16384, FF, dfk.DFK_BF16)
    wide.k2_splits = 16        # 16 blocks of 256 x 16384 fp32 exceed the partial-sum area (128 MiB)
    assert not dfk.dfk_config_valid(wide, 256, 16384, FF, dfk.DFK_BF16)
    assert dfk.dfk_config_valid(wide, 128, 16384, FF, dfk.DFK_BF16)


def test_candidates_and_workspace_over_random_shapes():
    """Host logic over a seeded sample of shapes: every candidate the scheduler lists is valid for its
    problem and passes the argument check with a workspace of the advertised size; there is always at
    least one; the workspace size is monotone in M; the untuned choice is one of the candidates."""
    import random
    rng = random.Random(20240611)
    fake = 1 << 30
    for _ in range(60):
        d = 8 * rng.choice([1, 2, 16, 33, 64, 128, 160, 512, 640, 1024])
        ff = 8 * rng.choice([1, 3, 33, 125, 352, 513, 1792, 3456, 3584])
        M = rng.choice([1, 2, 3, 7, 16, 17, 33, 64, 65, 100, 128, 200, 256])
        for dt in (dfk.DFK_BF16, dfk.DFK_FP16, dfk.DFK_FP32):
            n = dfk.dfk_num_candidates(M, d, ff, dt)
            assert n > 0, (M, d, ff, dt)
            wsb = dfk.dfk_workspace_bytes(M, d, ff)
            assert wsb >= dfk.dfk_workspace_bytes(max(1, M - 1), d, ff) > 0
            eb = 4 if dt == dfk.DFK_FP32 else 2
            nx, nw = M * d * eb, ff * d * eb
            al = lambda v: (v + 255) // 256 * 256
            Xp = fake; Wg = Xp + al(nx); Wu = Wg + al(nw); Wd = Wu + al(nw); Yp = Wd + al(nw); ws = Yp + al(nx)
            cands = []
            for i in range(n):
                c = dfk.dfk_get_candidate(M, d, ff, dt, i)
                cands.append(c.as_dict())
                assert dfk.dfk_config_valid(c, M, d, ff, dt), (M, d, ff, dt, c)
                assert dfk.dfk_check_args(Xp, Wg, Wu, Wd, Yp, M, d, ff, dt, c, ws, wsb) == dfk.DFK_OK, (M, d, ff, dt, c)
                if c.kmajor == 2:   # beyond 64 tokens, or where d_model rules the 64-token pair out
                    assert c.k2_col_blocks * 128 == d
                    assert M > 64 or d < 512
                if c.path == dfk.DFK_PATH_MFMA:
                    assert dt != dfk.DFK_FP32
            pick, tuned = dfk.dfk_get_choice(M, d, ff, dt)
            assert not tuned and pick.as_dict() in cands


def test_every_query_agrees_on_which_shapes_are_supported():
    """One token more than DFK_MAX_M, one step beyond the largest d_model, sizes that are not multiples
    of 8 or below 8: no candidates, no workspace or scratch size, no valid configuration, and the
    argument check says unsupported; at the limits themselves everything answers."""
    ok = dfk.dfk_get_candidate(4, 512, 512, dfk.DFK_BF16, 0)
    for dt in (dfk.DFK_BF16, dfk.DFK_FP16, dfk.DFK_FP32):
        for M, d, ff in ((dfk.DFK_MAX_M + 1, 512, 512), (4, 32768 + 8, 512), (4, 516, 512), (4, 512, 516), (4, 4, 512), (4, 512, 4)):
            assert dfk.dfk_num_candidates(M, d, ff, dt) == 0, (M, d, ff)
            assert dfk.dfk_workspace_bytes(M, d, ff) == 0, (M, d, ff)
            assert dfk.dfk_tune_scratch_bytes(M, d, ff, dt, 3) == 0, (M, d, ff)
            assert not dfk.dfk_config_valid(ok, M, d, ff, dt), (M, d, ff)
            with pytest.raises(dfk.DfkError) as ei:
                dfk.dfk_get_candidate(M, d, ff, dt, 0)
            assert ei.value.status == dfk.DFK_ERR_UNSUPPORTED_SHAPE
            with pytest.raises(dfk.DfkError) as ei:
                dfk.dfk_get_choice(M, d, ff, dt)
            assert ei.value.status == dfk.DFK_ERR_UNSUPPORTED_SHAPE
            assert dfk.dfk_check_args(X=X, W_gate=WG, W_up=WU, W_down=WD, Y=Y, M=M, d_model=d, d_ff=ff, dtype=dt) == dfk.DFK_ERR_UNSUPPORTED_SHAPE
        for M, d, ff in ((dfk.DFK_MAX_M, 32768, 8), (1, 8, 8), (dfk.DFK_MAX_M, 8, 262144)):
            n = dfk.dfk_num_candidates(M, d, ff, dt)
            assert n > 0, (M, d, ff)
            assert dfk.dfk_workspace_bytes(M, d, ff) > 0 and dfk.dfk_tune_scratch_bytes(M, d, ff, dt, 3) > 0
            c, _ = dfk.dfk_get_choice(M, d, ff, dt)
            assert dfk.dfk_config_valid(c, M, d, ff, dt)
            assert all(dfk.dfk_config_valid(dfk.dfk_get_candidate(M, d, ff, dt, i), M, d, ff, dt) for i in range(n))


def test_scheduler_table_roundtrip(tmp_path):
    dfk.dfk_clear_tuning()
    c0, tuned = dfk.dfk_get_choice(2, D, FF, dfk.DFK_BF16)
    assert not tuned and dfk.dfk_config_valid(c0, 2, D, FF, dfk.DFK_BF16)
    n = dfk.dfk_num_candidates(2, D, FF, dfk.DFK_BF16)
    pick = dfk.dfk_get_candidate(2, D, FF, dfk.DFK_BF16, n - 1)
    dfk.dfk_set_choice(2, D, FF, dfk.DFK_BF16, pick, 61.5)
    c1, tuned = dfk.dfk_get_choice(2, D, FF, dfk.DFK_BF16)
    assert tuned and c1.as_dict() == pick.as_dict()
    # a power-of-two bucket entry serves the M values below it
    pick8 = dfk.dfk_get_candidate(8, D, FF, dfk.DFK_BF16, 0)
    dfk.dfk_set_choice(8, D, FF, dfk.DFK_BF16, pick8, 70.0)
    c5, tuned5 = dfk.dfk_get_choice(5, D, FF, dfk.DFK_BF16)
    assert tuned5 and c5.as_dict() == pick8.as_dict()
    path = str(tmp_path / "tuning.txt")
    dfk.dfk_save_tuning(path)
    dfk.dfk_clear_tuning()
    assert not dfk.dfk_get_choice(2, D, FF, dfk.DFK_BF16)[1]
    dfk.dfk_load_tuning(path)
    c2, tuned = dfk.dfk_get_choice(2, D, FF, dfk.DFK_BF16)
    assert tuned and c2.as_dict() == pick.as_dict()
    # malformed file: error, table untouched
    with open(path, "a") as f:
        f.write("1 2 3 oops\n")
    with pytest.raises(dfk.DfkError) as ei:
        dfk.dfk_load_tuning(path)
    assert ei.value.status == dfk.DFK_ERR_IO
    assert dfk.dfk_get_choice(2, D, FF, dfk.DFK_BF16)[1]
    with pytest.raises(dfk.DfkError):
        dfk.dfk_load_tuning(str(tmp_path / "missing.txt"))
    dfk.dfk_clear_tuning()


def test_table_loader_survives_damaged_files(tmp_path):
    """Seeded damage to a saved table (fields replaced by huge, negative or non-numeric values, lines cut
    or doubled, binary bytes): loading either succeeds or reports an I/O error, and whatever the table
    then holds, the choice for a shape is a configuration that is valid for it."""
    import random
    rng = random.Random(99)
    dfk.dfk_clear_tuning()
    shapes = [(M, D, FF, dfk.DFK_BF16) for M in (1, 4, 64, 200)] + [(3, 512, 1000, dfk.DFK_FP32)]
    for M, d, ff, dt in shapes:
        n = dfk.dfk_num_candidates(M, d, ff, dt)
        dfk.dfk_set_choice(M, d, ff, dt, dfk.dfk_get_candidate(M, d, ff, dt, rng.randrange(n)), 50.0)
    good = str(tmp_path / "good.txt")
    dfk.dfk_save_tuning(good)
    lines = open(good).read().splitlines()
    junk = ["-1", "0", "7", "99999999999999999999", "2147483647", "-2147483648", "nan", "x", "", "1e9", "256", "3"]
    for case in range(300):
        out = []
        for ln in lines:
            r = rng.random()
            if ln.startswith("#") or r < 0.5:
                out.append(ln)
            elif r < 0.8:
                f = ln.split()
                f[rng.randrange(len(f))] = rng.choice(junk)
                out.append(" ".join(f))
            elif r < 0.9:
                out.append(ln[:rng.randrange(len(ln))])
            else:
                out.append(ln + " " + ln)
        path = str(tmp_path / "damaged.txt")
        with open(path, "wb") as f:
            f.write("\n".join(out).encode() + (bytes(rng.randrange(256) for _ in range(40)) if case % 7 == 0 else b"\n"))
        dfk.dfk_clear_tuning()
        try:
            dfk.dfk_load_tuning(path)
        except dfk.DfkError as e:
            assert e.status == dfk.DFK_ERR_IO
        for M, d, ff, dt in shapes:
            c, _ = dfk.dfk_get_choice(M, d, ff, dt)
            assert dfk.dfk_config_valid(c, M, d, ff, dt), (case, M, c)
    dfk.dfk_clear_tuning()


def test_timing_calls_check_their_arguments_on_the_host():
    import ctypes
    c = dfk.dfk_get_candidate(4, D, FF, dfk.DFK_BF16, 0)
    us = (ctypes.c_double * 2)()
    L = dfk.lib()
    fake = 256 * 4096    # never dereferenced: every case below fails before any HIP call
    assert L.dfk_time_kernels(None, 4, D, FF, 0, fake, 1 << 40, 2, 4, None, us) == dfk.DFK_ERR_INVALID_ARG
    assert L.dfk_time_kernels(ctypes.byref(c), 4, D, FF, 0, None, 1 << 40, 2, 4, None, us) == dfk.DFK_ERR_INVALID_ARG
    assert L.dfk_time_kernels(ctypes.byref(c), 4, D, FF, 0, fake, 1 << 40, 2, 0, None, us) == dfk.DFK_ERR_INVALID_ARG
    assert L.dfk_time_kernels(ctypes.byref(c), 4, D, FF, 0, fake, 1 << 40, 2, 4, None, None) == dfk.DFK_ERR_INVALID_ARG
    assert L.dfk_time_kernels(ctypes.byref(c), 4, D, FF, 0, fake + 8, 1 << 40, 2, 4, None, us) == dfk.DFK_ERR_ALIGNMENT
    assert L.dfk_time_kernels(ctypes.byref(c), 4, D, FF, 0, fake, 1024, 2, 4, None, us) == dfk.DFK_ERR_WORKSPACE
    # a token count that needs more than one set of launches cannot be split per kernel
    big = dfk.dfk_get_candidate(64, D, FF, dfk.DFK_BF16, 0)
    assert L.dfk_time_kernels(ctypes.byref(big), 64, D, FF, 0, fake, 1 << 40, 2, 4, None, us) == dfk.DFK_ERR_UNSUPPORTED_SHAPE


def test_helper_calls_check_their_arguments_on_the_host():
    L = dfk.lib()
    assert L.dfk_rms_normalize(None, 4096, 1, 512, None) == dfk.DFK_ERR_INVALID_ARG
    assert L.dfk_rms_normalize(4096, 4096, 0, 512, None) == dfk.DFK_ERR_INVALID_ARG
    assert L.dfk_rms_normalize(4096, 4096, 70000, 512, None) == dfk.DFK_ERR_UNSUPPORTED_SHAPE
    # the read-only kernel with the gate/up kernel's access pattern
    rp = L.dfk_read_gateup_pattern
    assert rp(None, WU, D, FF, 256, 8, WS, None) == dfk.DFK_ERR_INVALID_ARG
    assert rp(WG, WU, D, FF, 256, 8, None, None) == dfk.DFK_ERR_INVALID_ARG
    assert rp(WG, WU, D, FF, 256, 6, WS, None) == dfk.DFK_ERR_INVALID_ARG            # 4 or 8 wavefronts
    assert rp(WG, WU, D, FF, 0, 8, WS, None) == dfk.DFK_ERR_INVALID_ARG
    assert rp(WG, WU, D, FF, FF // 8 + 1, 8, WS, None) == dfk.DFK_ERR_UNSUPPORTED_SHAPE   # more slices than 8-row groups
    assert rp(WG, WU, D + 128, FF, 256, 8, WS, None) == dfk.DFK_ERR_UNSUPPORTED_SHAPE     # k range not whole 128-k chunks per wavefront
    assert rp(WG, WU, D, FF + 4, 256, 8, WS, None) == dfk.DFK_ERR_UNSUPPORTED_SHAPE
    assert rp(WG + 8, WU, D, FF, 256, 8, WS, None) == dfk.DFK_ERR_ALIGNMENT
    assert rp(WG, WU, D, FF, 256, 8, WS + 4, None) == dfk.DFK_ERR_ALIGNMENT


def test_mlp_block_checks_its_arguments_on_the_host():
    import ctypes
    L = dfk.lib()
    n = dfk.dfk_num_candidates(4, D, FF, dfk.DFK_BF16)
    cands = [dfk.dfk_get_candidate(4, D, FF, dfk.DFK_BF16, i) for i in range(n)]
    km = next(c for c in cands if c.kmajor == 1 and c.variant == dfk.DFK_VARIANT_TWO_KERNEL)
    other = next(c for c in cands if c.kmajor == 0)
    nx, nw = 4 * D * 2, FF * D * 2
    A = 1 << 30     # fake device addresses, never dereferenced: every case fails before any HIP call
    H, Wg, Wu, Wd, Y, w = A, A + (1 << 28), A + (2 << 28), A + (3 << 28), A + (4 << 28), A + (5 << 28)
    ws, wsb = A + (6 << 28), dfk.dfk_workspace_bytes(4, D, FF)

    def call(H=H, w=w, eps=1e-5, Wg=Wg, Y=Y, M=4, dtype=dfk.DFK_BF16, cfg=km, ws=ws, wsb=wsb):
        return L.dfk_mlp_block(H, w, eps, Wg, Wu, Wd, Y, M, D, FF, dtype, ctypes.byref(cfg) if cfg else None, ws, wsb, None)

    assert call(H=None) == dfk.DFK_ERR_INVALID_ARG
    assert call(w=None) == dfk.DFK_ERR_INVALID_ARG
    assert call(Y=None) == dfk.DFK_ERR_INVALID_ARG
    assert call(eps=-1.0) == dfk.DFK_ERR_INVALID_ARG
    assert call(eps=float("nan")) == dfk.DFK_ERR_INVALID_ARG
    assert call(dtype=7) == dfk.DFK_ERR_INVALID_ARG
    assert call(dtype=dfk.DFK_FP32) == dfk.DFK_ERR_UNSUPPORTED_SHAPE
    assert call(w=w + 2) == dfk.DFK_ERR_ALIGNMENT
    assert call(Y=H + 16) == dfk.DFK_ERR_ALIAS            # partial overlap with the input
    assert call(Y=Wg) == dfk.DFK_ERR_ALIAS
    assert call(w=Y + 64) == dfk.DFK_ERR_ALIAS
    assert call(ws=None) == dfk.DFK_ERR_WORKSPACE
    assert call(wsb=1024) == dfk.DFK_ERR_WORKSPACE
    assert call(cfg=other) == dfk.DFK_ERR_UNSUPPORTED_SHAPE   # only the kernel pair for up to 64 tokens carries it
    assert call(M=0) == dfk.DFK_ERR_INVALID_ARG


def test_status_strings():
    for s in range(0, -9, -1):
        assert dfk.dfk_status_string(s) not in ("", "unknown status")
    assert dfk.dfk_status_string(-99) == "unknown status"


def test_static_scratch_entry_point_rejects_on_the_host():
    """dfk_swiglu_mlp_static checks its arguments and its size limits before any HIP call."""
    l = dfk.lib()
    call = lambda M, d, ff, x=X, cfg=None: l.dfk_swiglu_mlp_static(x, WG, WU, WD, Y, M, d, ff, dfk.DFK_BF16, cfg, None)
    assert call(1, D, FF, x=0) == dfk.DFK_ERR_INVALID_ARG
    assert call(0, D, FF) == dfk.DFK_ERR_INVALID_ARG
    assert call(1, 4100, FF) == dfk.DFK_ERR_UNSUPPORTED_SHAPE
    assert call(1, D, FF, x=X + 8) == dfk.DFK_ERR_ALIGNMENT
    # A_2 of M x d_ff fp32 beyond its 16 MiB share of the array
    assert call(256, 512, 16392) == dfk.DFK_ERR_WORKSPACE
    assert call(16, 8, 262152) == dfk.DFK_ERR_WORKSPACE
    # an explicit configuration whose partial sums do not fit what is left (512 slices x 8 tokens x 8192 columns of fp32: 128 MiB)
    big = None
    for i in range(dfk.dfk_num_candidates(8, 8192, 8192, dfk.DFK_BF16)):
        c = dfk.dfk_get_candidate(8, 8192, 8192, dfk.DFK_BF16, i)
        if c.variant == dfk.DFK_VARIANT_FUSED and c.path == dfk.DFK_PATH_VALU and c.splits == 512:
            big = c
    assert big is not None
    assert call(8, 8192, 8192, cfg=ctypes.byref(big)) == dfk.DFK_ERR_WORKSPACE


def test_valu_configuration_at_the_lds_boundary_is_refused_on_the_host():
    """The VALU kernels keep MT x slice rows of fp32 in dynamic LDS under the default 64 KiB allowance,
    next to a static word: a configuration that needs the full 64 KiB must fail the host check, not the launch."""
    c = dfk.dfk_get_candidate(8, 512, 16384, dfk.DFK_BF16, 0)
    c.variant, c.path, c.kmajor, c.k2_rows_by_wave, c.reduce = dfk.DFK_VARIANT_FUSED, dfk.DFK_PATH_VALU, 0, 0, dfk.DFK_REDUCE_TICKET
    c.waves, c.depth, c.k2_splits, c.k2_col_blocks = 8, 0, 0, 0
    c.splits = 8                       # 8 tokens x 2048 rows = 16384 floats = 64 KiB exactly
    assert not dfk.dfk_config_valid(c, 8, 512, 16384, dfk.DFK_BF16)
    c.splits = 16                      # 8 x 1024 floats = 32 KiB
    assert dfk.dfk_config_valid(c, 8, 512, 16384, dfk.DFK_BF16)


def test_tune_skip_report_starts_empty():
    n, status = dfk.dfk_tune_skipped()
    assert n == 0 and status == dfk.DFK_OK


def test_a_configuration_belongs_to_one_layout_of_w_down(tmp_path):
    """The kernels for W_down given as [d_model, d_ff] (kmajor = 5) are listed, chosen, stored and called apart
    from the others; every mix-up is refused on the host, before any HIP call."""
    import ctypes
    L = dfk.lib()
    dfk.dfk_clear_tuning()
    n = dfk.dfk_workspace_bytes(16, D, FF)
    wdt = [dfk.dfk_get_candidate_wdt(16, D, FF, dfk.DFK_BF16, i) for i in range(dfk.dfk_num_candidates_wdt(16, D, FF, dfk.DFK_BF16))]
    plain = [dfk.dfk_get_candidate(16, D, FF, dfk.DFK_BF16, i) for i in range(dfk.dfk_num_candidates(16, D, FF, dfk.DFK_BF16))]
    assert wdt and all(c.kmajor == 5 and dfk.dfk_config_valid(c, 16, D, FF, dfk.DFK_BF16) for c in wdt)
    assert all(c.kmajor != 5 for c in plain)
    args = (X, WG, WU, WD, Y, 16, D, FF, dfk.DFK_BF16)
    # the wrong kind of configuration for an entry point
    assert L.dfk_swiglu_mlp_ex(*args, ctypes.byref(wdt[0]), WS, n, None) == dfk.DFK_ERR_INVALID_ARG
    assert L.dfk_swiglu_mlp_static(*args, ctypes.byref(wdt[0]), None) == dfk.DFK_ERR_INVALID_ARG
    assert L.dfk_check_args(*args, ctypes.byref(wdt[0]), WS, n) == dfk.DFK_ERR_INVALID_ARG
    assert L.dfk_swiglu_mlp_wdt(*args, ctypes.byref(plain[0]), WS, n, None) == dfk.DFK_ERR_INVALID_ARG
    # argument checks of the entry point itself
    assert L.dfk_swiglu_mlp_wdt(X, WG, WU, None, Y, 16, D, FF, dfk.DFK_BF16, None, WS, n, None) == dfk.DFK_ERR_INVALID_ARG
    assert L.dfk_swiglu_mlp_wdt(*args, None, None, 0, None) == dfk.DFK_ERR_WORKSPACE
    assert L.dfk_swiglu_mlp_wdt(*args, None, WS, n - 1, None) == dfk.DFK_ERR_WORKSPACE
    assert L.dfk_swiglu_mlp_wdt(X, WG, WU, WD + 8, Y, 16, D, FF, dfk.DFK_BF16, None, WS, n, None) == dfk.DFK_ERR_ALIGNMENT
    assert L.dfk_swiglu_mlp_wdt(X, WG, WU, Y, Y, 16, D, FF, dfk.DFK_BF16, None, WS, n, None) == dfk.DFK_ERR_ALIAS
    # shapes and types the MFMA kernels of this layout do not take are served by its plain-FMA pair
    for M_, d_, ff_, dt_ in ((16, D, FF, dfk.DFK_FP32), (16, D, FF + 8, dfk.DFK_BF16), (16, 264, 1024, dfk.DFK_BF16),
                             (16, 4096, 384, dfk.DFK_BF16)):   # (fewer 128-k chunks of d_ff than wavefronts)
        cs = [dfk.dfk_get_candidate_wdt(M_, d_, ff_, dt_, i) for i in range(dfk.dfk_num_candidates_wdt(M_, d_, ff_, dt_))]
        assert cs and all(c.kmajor == 5 and c.path == dfk.DFK_PATH_VALU for c in cs)
        assert dfk.dfk_get_choice_wdt(M_, d_, ff_, dt_)[0].as_dict() == cs[0].as_dict()
        assert L.dfk_swiglu_mlp_ex(X, WG, WU, WD, Y, M_, d_, ff_, dt_, ctypes.byref(cs[0]), WS, 1 << 40, None) == dfk.DFK_ERR_INVALID_ARG
    # where both exist the MFMA pair comes first (the untuned default)
    assert wdt[0].path == dfk.DFK_PATH_MFMA and wdt[-1].path == dfk.DFK_PATH_VALU
    # unsupported shapes stay unsupported
    assert dfk.dfk_num_candidates_wdt(16, 4100, FF, dfk.DFK_BF16) == 0
    assert L.dfk_swiglu_mlp_wdt(X, WG, WU, WD, Y, 16, 4100, FF, dfk.DFK_BF16, None, WS, 1 << 40, None) == dfk.DFK_ERR_UNSUPPORTED_SHAPE
    # the table keeps the layouts apart, also through a file
    pick, tuned = dfk.dfk_get_choice_wdt(16, D, FF, dfk.DFK_BF16)
    assert not tuned and pick.as_dict() == wdt[0].as_dict()
    dfk.dfk_set_choice(16, D, FF, dfk.DFK_BF16, wdt[-1], 60.0)
    dfk.dfk_set_choice(16, D, FF, dfk.DFK_BF16, plain[3], 61.0)
    assert dfk.dfk_get_choice_wdt(16, D, FF, dfk.DFK_BF16)[0].as_dict() == wdt[-1].as_dict()
    assert dfk.dfk_get_choice(16, D, FF, dfk.DFK_BF16)[0].as_dict() == plain[3].as_dict()
    path = str(tmp_path / "tuning.txt")
    dfk.dfk_save_tuning(path)
    dfk.dfk_clear_tuning()
    dfk.dfk_load_tuning(path)
    got, tuned = dfk.dfk_get_choice_wdt(16, D, FF, dfk.DFK_BF16)
    assert tuned and got.as_dict() == wdt[-1].as_dict()
    got, tuned = dfk.dfk_get_choice(16, D, FF, dfk.DFK_BF16)
    assert tuned and got.as_dict() == plain[3].as_dict()
    dfk.dfk_clear_tuning()
    # the transpose helper
    tr = L.dfk_transpose_w_down
    assert tr(None, WD, D, FF, dfk.DFK_BF16, None) == dfk.DFK_ERR_INVALID_ARG
    assert tr(WD, WD + 2 * A, 0, FF, dfk.DFK_BF16, None) == dfk.DFK_ERR_INVALID_ARG
    assert tr(WD, WD + 2 * A, D, FF, 9, None) == dfk.DFK_ERR_INVALID_ARG
    assert tr(WD + 4, WD + 2 * A, D, FF, dfk.DFK_BF16, None) == dfk.DFK_ERR_ALIGNMENT
    assert tr(WD, WD + 4096, D, FF, dfk.DFK_BF16, None) == dfk.DFK_ERR_ALIAS
