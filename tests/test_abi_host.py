"""CPU-only: the C-ABI library loads, exports every symbol the header declares, and its host-side
logic (la table, workspace size, error strings, argument checks) behaves as documented.  No kernel
is launched here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2501_16376_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2501_16376_amd import build
        build.build_library()
    return binding.load_library()


def test_exports_match_header(lib):
    text = open(os.path.join(ROOT, "include", "swiftprune.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(swiftprune_\w+)\s*\(", text))
    assert {"swiftprune_layer_stats", "swiftprune_score_select", "swiftprune_nm_select",
            "swiftprune_apply"} <= declared
    for name in declared:
        assert hasattr(lib, name), f"{name} is declared in the header but not exported"
    from paper_2501_16376_amd import binding
    assert set(binding.EXPORTS) == declared


def test_header_is_plain_c_and_links(lib, tmp_path):
    """The header compiles as C11 and as C++17 with warnings as errors, and a plain-C caller links against
    the library and gets the documented host-side answers (no device call is made)."""
    import subprocess
    from paper_2501_16376_amd import binding
    inc = os.path.join(ROOT, "include")
    src = tmp_path / "caller.c"
    src.write_text(
        '#include "swiftprune.h"\n#include <stdio.h>\n'
        "int main(void) {\n"
        "    float la = 0.0f;\n"
        "    sp_ewma_params p = {0.125f, 0.125f, 0.5f};\n"
        "    if (swiftprune_la_for_sparsity(0.7f, &la) != SP_OK || la != -0.2f) return 1;\n"
        "    if (swiftprune_layer_stats(NULL, 1, 1, 1, SP_F16, NULL, NULL, NULL, 0, 1, NULL, 0, NULL) != SP_EINVAL) return 2;\n"
        "    if (swiftprune_nm_meta_words(4096, 2, 4) != 128) return 3;\n"
        '    printf("%s %zu %g\\n", swiftprune_version(), swiftprune_stats_workspace_bytes(262144, 4096), (double)p.la);\n'
        "    return 0;\n}\n")
    subprocess.run(["gcc", "-std=c11", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", inc, "-c", str(src),
                    "-o", str(tmp_path / "caller.o")], check=True)
    subprocess.run(["g++", "-std=c++17", "-Wall", "-Wextra", "-Werror", "-I", inc, "-x", "c++", "-fsyntax-only",
                    os.path.join(inc, "swiftprune.h")], check=True)
    lib_dir = os.path.dirname(binding.LIB_PATH)
    exe = tmp_path / "caller"
    subprocess.run(["gcc", str(tmp_path / "caller.o"), "-o", str(exe), "-L", lib_dir, "-lswiftprune",
                    f"-Wl,-rpath,{lib_dir}", "-Wl,-rpath,/opt/rocm/lib"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert out[0] == "0.1.0" and int(out[1]) > 0 and float(out[2]) == 0.5


def test_version_and_strerror(lib):
    from paper_2501_16376_amd import binding
    assert re.match(r"^\d+\.\d+\.\d+$", binding.swiftprune_version())
    assert binding.swiftprune_strerror(0) == "success"
    for code in (-1, -2, -3, -99):
        assert binding.swiftprune_strerror(code)


def test_la_table_matches_paper(lib):
    """Exact values of the paper's ratio -> la table (tests/golden/la_table.txt), linear in between."""
    from paper_2501_16376_amd import binding
    rows = [l.split() for l in open(os.path.join(ROOT, "tests", "golden", "la_table.txt"))
            if l.strip() and not l.startswith("#")]
    table = {int(r[0]): float(r[1]) for r in rows}
    assert table == {90: -1.5, 80: -0.9, 70: -0.2, 60: 0.2, 50: 0.5}
    for pct, la in table.items():
        assert binding.swiftprune_la_for_sparsity(pct / 100.0) == pytest.approx(la, abs=1e-7)
    assert binding.swiftprune_la_for_sparsity(0.55) == pytest.approx(0.35, abs=1e-6)
    assert binding.swiftprune_la_for_sparsity(0.75) == pytest.approx(-0.55, abs=1e-6)
    for bad in (0.3, 0.49, 0.91, 1.0, float("nan")):
        with pytest.raises(binding.SwiftPruneError):
            binding.swiftprune_la_for_sparsity(bad)
    assert lib.swiftprune_la_for_sparsity(0.5, None) == binding.SP_EINVAL


def test_workspace_bytes(lib):
    from paper_2501_16376_amd import binding
    assert binding.swiftprune_stats_workspace_bytes(0, 4096) == 0
    assert binding.swiftprune_stats_workspace_bytes(128, -1) == 0
    for tokens, n in [(1, 1), (128, 256), (262144, 4096), (262144, 11008), (262144, 14336), (262144, 28672)]:
        b = binding.swiftprune_stats_workspace_bytes(tokens, n)
        assert 256 < b < 64 << 20, (tokens, n, b)      # a header plus at most a few MB of partial rows


def test_argument_checks_do_not_launch(lib):
    """Bad arguments are refused on the host (SP_EINVAL / SP_ENOSPC) before any HIP call."""
    from paper_2501_16376_amd import binding
    p = 0x10000                                        # never dereferenced: checks fail first
    ws = 1 << 20
    E = binding.SP_EINVAL
    st = lib.swiftprune_layer_stats
    assert st(None, 8, 8, 8, 1, p, p, p, 0, 1, p, ws, None) == E
    assert st(p, 0, 8, 8, 1, p, p, p, 0, 1, p, ws, None) == E
    assert st(p, 8, -1, 8, 1, p, p, p, 0, 1, p, ws, None) == E
    assert st(p, 8, 8, 7, 1, p, p, p, 0, 1, p, ws, None) == E          # pitch < columns
    assert st(p, 8, 8, 8, 7, p, p, p, 0, 1, p, ws, None) == E          # unknown dtype
    assert st(p, 8, 8, 8, 1, p, None, p, 0, 1, p, ws, None) == E       # finalize needs S
    assert st(p, 8, 8, 8, 1, p, p, p, 0, 1, p + 8, ws, None) == E      # workspace alignment
    assert st(p, 262144, 4096, 4096, 1, p, p, p, 0, 1, p, 1024, None) == binding.SP_ENOSPC
    sel = lib.swiftprune_score_select
    prm = binding.sp_ewma_params(0.125, 0.125, 0.5)
    assert sel(None, 8, 8, 8, 1, p, 0.5, C.byref(prm), p, None, None, 0, None) == E
    assert sel(p, 8, 8, 8, 1, None, 0.5, C.byref(prm), p, None, None, 0, None) == E
    assert sel(p, 8, 8, 8, 1, p, 0.5, C.byref(prm), None, None, None, 0, None) == E
    assert sel(p, 8, 8, 4, 1, p, 0.5, C.byref(prm), p, None, None, 0, None) == E
    assert sel(p, 8, 8, 8, 1, p, 0.5, C.byref(prm), p, None, None, 64, None) == E      # unknown flag
    for bad in (binding.sp_ewma_params(0.0, 0.125, 0.5), binding.sp_ewma_params(0.125, 1.5, 0.5),
                binding.sp_ewma_params(float("nan"), 0.125, 0.5),
                binding.sp_ewma_params(0.125, 0.125, float("inf"))):
        assert sel(p, 8, 8, 8, 1, p, 0.5, C.byref(bad), p, None, None, 0, None) == E
    nanla = binding.sp_ewma_params(0.125, 0.125, float("nan"))
    assert sel(p, 8, 8, 8, 1, p, 0.3, C.byref(nanla), p, None, None, 0, None) == E     # no la for 0.3
    nm = lib.swiftprune_nm_select
    assert nm(p, 8, 8, 8, 1, p, 2, 5, p, None, 0, None) == E          # unsupported group size
    assert nm(p, 8, 8, 8, 1, p, 4, 4, p, None, 0, None) == E          # n_keep must be < m
    assert nm(p, 8, 8, 8, 1, p, 0, 4, p, None, 0, None) == E
    assert nm(p, 8, 12, 12, 1, p, 4, 8, p, None, 0, None) == E        # in % m != 0
    assert nm(p, 8, 8, 8, 1, p, 2, 4, p, None, 1, None) == E          # strict-order flag not valid here
    grp, ngrp = lib.swiftprune_score_select_group, lib.swiftprune_nm_select_group
    ok = binding.sp_matrix(p, 8, 8, p, None)
    two = (binding.sp_matrix * 2)(ok, ok)
    assert grp(None, 1, 8, 1, p, 0.5, C.byref(prm), 0, None) == E
    assert grp(two, 0, 8, 1, p, 0.5, C.byref(prm), 0, None) == E
    assert grp(two, 9, 8, 1, p, 0.5, C.byref(prm), 0, None) == E             # more than SP_MAX_GROUP
    assert grp(two, 2, 8, 1, None, 0.5, C.byref(prm), 0, None) == E
    assert grp(two, 2, 8, 1, p, 0.5, C.byref(prm), 64, None) == E
    assert grp(two, 2, 8, 1, p, 0.3, C.byref(nanla), 0, None) == E
    for broken in (binding.sp_matrix(None, 8, 8, p, None), binding.sp_matrix(p, 0, 8, p, None),
                   binding.sp_matrix(p, 8, 7, p, None), binding.sp_matrix(p, 8, 8, None, None),
                   binding.sp_matrix(p + 1, 8, 8, p, None)):
        arr = (binding.sp_matrix * 2)(ok, broken)
        assert grp(arr, 2, 8, 1, p, 0.5, C.byref(prm), 0, None) == E
        assert ngrp(arr, 2, 8, 1, p, 2, 4, 0, None) == E
    assert ngrp(two, 2, 8, 1, p, 2, 5, 0, None) == E
    assert ngrp(two, 2, 12, 1, p, 4, 8, 0, None) == E                        # in % m != 0 (and pitch < columns)
    assert ngrp(two, 2, 8, 1, p, 2, 4, 1, None) == E
    cf = lib.swiftprune_channel_factor
    assert cf(None, p, 8, p, None) == E and cf(p, None, 8, p, None) == E and cf(p, p, 8, None, None) == E
    assert cf(p, p, 0, p, None) == E and cf(p + 2, p, 8, p, None) == E
    fp = lib.swiftprune_layer_stats_from_partials
    assert fp(None, 4, 8, 8, p, p, p, 0, 1, None) == E and fp(p, 4, 8, 8, None, p, p, 0, 1, None) == E
    assert fp(p, 4, 8, 8, p, None, p, 0, 1, None) == E and fp(p, 4, 8, 8, p, p, None, 0, 1, None) == E   # finalize needs hr
    assert fp(p, 0, 8, 8, p, p, p, 0, 1, None) == E and fp(p, 4, 0, 8, p, p, p, 0, 1, None) == E
    assert fp(p, 4, 8, 7, p, p, p, 0, 1, None) == E                          # pitch < columns
    assert fp(p + 2, 4, 8, 8, p, p, p, 0, 1, None) == E and fp(p, (1 << 24) + 1, 8, 8, p, p, p, 0, 1, None) == E
    tr = lib.swiftprune_ewma_trace
    assert tr(p, 8, 8, 8, 1, p, 0.125, 0.125, None, None, None) == E         # nothing to write
    assert tr(None, 8, 8, 8, 1, p, 0.125, 0.125, p, p, None) == E
    assert tr(p, 8, 8, 8, 1, p, 0.0, 0.125, p, p, None) == E
    assert tr(p, 8, 8, 8, 1, p, 0.125, 0.125, p + 2, p, None) == E           # misaligned float pointer
    cp = lib.swiftprune_count_pruned
    las = (C.c_float * 3)(0.5, 0.2, -0.2)
    assert cp(p, 8, 8, 8, 1, p, 0.125, 0.125, las, 0, p, None) == E          # n_la < 1
    assert cp(p, 8, 8, 8, 1, p, 0.125, 0.125, las, 17, p, None) == E         # n_la > 16
    assert cp(p, 8, 8, 8, 1, p, 0.125, 0.125, None, 3, p, None) == E
    assert cp(p, 8, 8, 8, 1, p, 0.125, 0.125, las, 3, p + 4, None) == E      # counts alignment
    bad = (C.c_float * 2)(0.5, float("nan"))
    assert cp(p, 8, 8, 8, 1, p, 0.125, 0.125, bad, 2, p, None) == E
    cal = lib.swiftprune_calibrate_la
    la_o, ach_o = C.c_float(), C.c_float()
    assert cal(p, 8, 8, 8, 1, p, 0.125, 0.125, 0.0, 1e-3, -8.0, 8.0, p, C.byref(la_o), C.byref(ach_o), None) == E
    assert cal(p, 8, 8, 8, 1, p, 0.125, 0.125, 0.3, 0.0, -8.0, 8.0, p, C.byref(la_o), C.byref(ach_o), None) == E
    assert cal(p, 8, 8, 8, 1, p, 0.125, 0.125, 0.3, 1e-3, 2.0, 1.0, p, C.byref(la_o), C.byref(ach_o), None) == E
    assert cal(p, 8, 8, 8, 1, p, 0.125, 0.125, 0.3, 1e-3, -8.0, 8.0, None, C.byref(la_o), C.byref(ach_o), None) == E
    cd = lib.swiftprune_calibrate_la_device
    wsb = lib.swiftprune_la_workspace_bytes()
    assert 8192 <= wsb <= 65536
    assert cd(None, 8, 8, 8, 1, p, 0.125, 0.125, 0.3, p, wsb, p, None, None, None) == E
    assert cd(p, 8, 8, 8, 1, p, 0.125, 0.125, 0.0, p, wsb, p, None, None, None) == E
    assert cd(p, 8, 8, 8, 1, p, 0.125, 0.125, 1.0, p, wsb, p, None, None, None) == E
    assert cd(p, 8, 8, 8, 1, p, 0.125, 0.125, 0.3, p + 8, wsb, p, None, None, None) == E   # workspace alignment
    assert cd(p, 8, 8, 8, 1, p, 0.125, 0.125, 0.3, p, wsb, None, None, None, None) == E
    assert cd(p, 8, 8, 8, 1, p, 0.125, 0.125, 0.3, p, wsb, p, p + 4, None, None) == E      # uint64 alignment
    assert cd(p, 8, 8, 8, 1, p, 0.125, 0.125, 0.3, p, 16, p, None, None, None) == binding.SP_ENOSPC
    sl = lib.swiftprune_score_select_la
    assert sl(p, 8, 8, 8, 1, p, 0.125, 0.125, None, p, None, 0, None) == E
    assert sl(p, 8, 8, 8, 1, p, 0.125, 0.125, p, None, None, 0, None) == E
    assert sl(p, 8, 8, 8, 1, p, 0.125, 0.125, p, p, None, 1, None) == E                    # strict-order flag not valid here
    assert sl(p, 8, 8, 8, 1, p, 0.0, 0.125, p, p, None, 0, None) == E
    tk = lib.swiftprune_topk_select
    assert tk(None, 8, 8, 8, 1, p, None, 4, p, 0, None) == E
    assert tk(p, 8, 8, 8, 1, p, None, 4, None, 0, None) == E
    assert tk(p, 8, 8, 8, 1, p, None, 4, p, 1, None) == E                    # strict-order flag not valid here
    cn = lib.swiftprune_compact_nm
    assert cn(p, 8, 8, 8, 1, p, 2, 4, None, p, None) == E
    assert cn(p, 8, 8, 8, 1, p, 2, 5, p, p, None) == E
    assert cn(p, 8, 12, 12, 1, p, 4, 8, p, p, None) == E
    ex = lib.swiftprune_expand_nm
    assert ex(p, p, 8, 8, 1, 2, 4, p, 4, None) == E                          # pitch < columns
    assert ex(p, None, 8, 8, 1, 2, 4, p, 8, None) == E
    assert lib.swiftprune_nm_meta_words(4096, 2, 4) == 128 and lib.swiftprune_nm_meta_words(4096, 4, 8) == 256
    assert lib.swiftprune_nm_meta_words(4096, 2, 5) == 0 and lib.swiftprune_nm_meta_words(10, 2, 4) == 0
    ap = lib.swiftprune_apply
    assert ap(None, 8, 8, 8, 1, p, None) == E
    assert ap(p, 8, 8, 8, 1, None, None) == E
    assert ap(p + 1, 8, 8, 8, 1, p, None) == E                        # misaligned element pointer


def test_binding_refuses_cpu_tensors(lib):
    import torch
    from paper_2501_16376_amd import binding
    W = torch.zeros(4, 8, dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        binding.swiftprune_apply(W, torch.zeros(4, 1, dtype=torch.int32))


def test_missing_library_fails_loudly(tmp_path):
    from paper_2501_16376_amd import binding
    with pytest.raises(ImportError):
        binding.load_library(str(tmp_path / "nope.so"))


def test_synth_bf16_roundtrip():
    """The bf16 storage helpers round to nearest-even and widen exactly (checked against torch)."""
    import torch
    from paper_2501_16376_amd import synth
    a = np.random.default_rng(0).standard_normal(10000).astype(np.float32) * 3
    bits = synth.f32_to_bf16_bits(a)
    ref = torch.from_numpy(a).to(torch.bfloat16)
    assert np.array_equal(bits, ref.view(torch.int16).numpy().view(np.uint16))
    assert np.array_equal(synth.bf16_bits_to_f32(bits), ref.to(torch.float32).numpy())
    W, X = synth.config1()
    assert W.shape == (256, 256) and X.shape == (128, 256) and W.dtype == np.float32
    assert abs(float(W.std()) - 0.02) < 1e-3
