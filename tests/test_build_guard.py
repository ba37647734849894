"""Host-side build logic (CPU only)."""
from paper_2412_18106_amd import build as B


def test_scratch_report_reads_the_compiler_remarks():
    text = ("a.hip:1:1: remark: Function Name: kernel_a [-Rpass-analysis=kernel-resource-usage]\n"
            "a.hip:1:1: remark:     VGPRs: 12 [-Rpass-analysis=kernel-resource-usage]\n"
            "a.hip:1:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]\n"
            "a.hip:9:1: remark: Function Name: kernel_b [-Rpass-analysis=kernel-resource-usage]\n"
            "a.hip:9:1: remark:     ScratchSize [bytes/lane]: 148 [-Rpass-analysis=kernel-resource-usage]\n")
    assert B._scratch_report(text) == {"kernel_a": 0, "kernel_b": 148}
    assert B._scratch_report("") == {}


def test_hazard_lint_flags_reads_of_hand_issued_results_and_passes_padded_code():
    from paper_2412_18106_amd import hazard_lint as H
    bad = """
	;;#ASMSTART
	v_mfma_f32_32x32x16_bf16 v[18:33], v[98:101], v[146:149], v[18:33]
	;;#ASMEND
	v_mov_b64_e32 v[112:113], v[48:49]
	v_mov_b64_e32 v[128:129], v[32:33]
"""
    assert len(H.lint(bad)) == 1 and "v[32:33]" in H.lint(bad)[0][1]
    good = """
	;;#ASMSTART
	v_mfma_f32_32x32x16_bf16 v[18:33], v[98:101], v[146:149], v[18:33]
	;;#ASMEND
	;;#ASMSTART
	s_nop 7
	s_nop 4
	;;#ASMEND
	v_mov_b64_e32 v[128:129], v[32:33]
"""
    assert H.lint(good) == []
    chain = """
	;;#ASMSTART
	v_mfma_f32_32x32x16_bf16 v[18:33], v[98:101], v[146:149], v[18:33]
	;;#ASMEND
	;;#ASMSTART
	v_mfma_f32_32x32x16_bf16 v[18:33], v[102:105], v[146:149], v[18:33]
	;;#ASMEND
.LBB0_3:
	v_add_f32_e32 v18, v18, v1
"""
    assert H.lint(chain) == []          # MFMAs order themselves; past the label nothing is claimed
    lds = """
	;;#ASMSTART
	ds_read_b128 v[82:85], v82 offset:0
	;;#ASMEND
	scratch_store_dwordx4 off, v[82:85], off offset:76
"""
    assert len(H.lint(lds)) == 1
    lds_ok = """
	;;#ASMSTART
	ds_read_b128 v[82:85], v90 offset:0
	;;#ASMEND
	v_add_f32_e32 v1, v2, v3
	;;#ASMSTART
	s_waitcnt lgkmcnt(0)
	;;#ASMEND
	v_mov_b32_e32 v5, v82
"""
    assert H.lint(lds_ok) == []


def test_hazard_lint_flags_compiler_writes_right_in_front_of_a_hand_issued_mfma():
    from paper_2412_18106_amd import hazard_lint as H
    # a constant the compiler rebuilt next to the MFMA that reads it (seen on the GPU as stale operand data)
    bad = """
	v_mov_b64_e32 v[16:17], s[10:11]
	v_mov_b64_e32 v[14:15], s[8:9]
	;;#ASMSTART
	v_mfma_f32_32x32x16_bf16 a[0:15], v[18:21], v[14:17], a[0:15]
	;;#ASMEND
"""
    found = H.lint(bad)
    assert len(found) == 1 and "reads a register" in found[0][1]
    padded = """
	v_mov_b64_e32 v[14:15], s[8:9]
	;;#ASMSTART
	s_nop 4
	;;#ASMEND
	;;#ASMSTART
	v_mfma_f32_32x32x16_bf16 a[0:15], v[18:21], v[14:17], a[0:15]
	;;#ASMEND
"""
    assert H.lint(padded) == []
    # accumulation registers are tracked as well, apart from the vector registers of the same number
    agpr = """
	v_accvgpr_write_b32 a3, v7
	;;#ASMSTART
	v_mfma_f32_32x32x16_bf16 v[32:47], v[110:113], a[0:3], v[66:81]
	;;#ASMEND
"""
    assert len(H.lint(agpr)) == 1
    other_file = """
	v_mov_b32_e32 v3, v7
	;;#ASMSTART
	v_mfma_f32_32x32x16_bf16 v[32:47], v[110:113], a[0:3], v[66:81]
	;;#ASMEND
"""
    assert H.lint(other_file) == []
    # what another inline-assembly statement wrote is the author's business, not the compiler's
    own = """
	;;#ASMSTART
	v_mov_b32_e32 v110, v7
	;;#ASMEND
	;;#ASMSTART
	v_mfma_f32_32x32x16_bf16 v[32:47], v[110:113], a[0:3], v[66:81]
	;;#ASMEND
"""
    assert H.lint(own) == []


def test_hazard_lint_flags_an_inline_scalar_instruction_between_a_compare_and_its_branch():
    """An inline-assembly statement that writes SCC without saying so: the compiler keeps its loop compare live
    across it and the branch reads the statement's flag instead."""
    from paper_2412_18106_amd import hazard_lint
    bad = """
.LBB0_1:
\ts_load_dword s24, s[26:27], 0x0
\ts_cmpk_eq_i32 s22, 0x80
\ts_waitcnt lgkmcnt(0)
\t;;#ASMSTART
\ts_and_b32 s24, s24, 0
\t;;#ASMEND
\ts_cbranch_scc0 .LBB0_1
"""
    found = hazard_lint.lint(bad)
    assert len(found) == 1 and "SCC" in found[0][1] and found[0][0] == 9
    good = """
.LBB0_1:
\ts_load_dword s24, s[26:27], 0x0
\ts_waitcnt lgkmcnt(0)
\t;;#ASMSTART
\ts_and_b32 s24, s24, 0
\t;;#ASMEND
\ts_cmpk_eq_i32 s22, 0x80
\ts_cbranch_scc0 .LBB0_1
"""
    assert hazard_lint.lint(good) == []
    # an inline statement that only waits or moves does not write the flag
    harmless = bad.replace("s_and_b32 s24, s24, 0", "s_nop 4")
    assert hazard_lint.lint(harmless) == []


def test_gap_tables_in_the_kernel_source_are_the_generated_ones():
    """The placement tables of the wide iteration are made by gap_tables.py; the source must carry what it prints,
    and the tables must obey the ordering rules (no packing or addition in the gap of an exponential it reads)."""
    import os
    import re
    from paper_2412_18106_amd import gap_tables as G
    ke, kc, ka = G.tables()
    G.check(ke, kc, ka)
    assert max(G.gap_costs(ke, kc, ka)) <= G.GAP_CAP
    src = open(os.path.join(os.path.dirname(G.__file__), "csrc", "attn_kernels.hip")).read()
    for name, table in (("EXP", ke), ("CVT", kc), ("ADD", ka)):
        m = re.search(r"#define XY_GAP_TABLE_%s \{([^}]*)\}" % name, src)
        assert m and [int(x) for x in m.group(1).split(",")] == table, name
    # a table that breaks the rule is refused
    bad = list(kc)
    bad[1] = 1
    try:
        G.check(ke, bad, ka)
    except AssertionError:
        pass
    else:
        raise AssertionError("a packing in the gap of its own exponentials was accepted")


def test_library_stamp_tells_a_current_library_from_a_stale_one(tmp_path, monkeypatch):
    """The build writes the digest of the sources next to the library; the binding loads the library only when
    the digest of the tree still equals it."""
    assert B.is_current()                       # the suite runs against a library built from this tree
    assert B.sources_digest() == B.sources_digest() and len(B.sources_digest()) == 64
    stamp = tmp_path / "stamp"
    monkeypatch.setattr(B, "STAMP", str(stamp))
    assert not B.is_current()                   # no stamp: unknown origin
    stamp.write_text("0" * 64 + "\n")
    assert not B.is_current()                   # built from something else
    stamp.write_text(B.sources_digest() + "\n")
    assert B.is_current()


def test_product_and_oracle_do_not_know_each_other():
    """No module of the package imports the oracle (the product path never routes through it), no module of the
    oracle imports the package, and in bench.py and the entry script the oracle is touched only by the baseline
    leg and the smoke check."""
    import ast
    import glob
    import os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

    def imported(path):
        names = set()
        for node in ast.walk(ast.parse(open(path).read())):
            if isinstance(node, ast.Import):
                names.update(a.name.split(".")[0] for a in node.names)
            elif isinstance(node, ast.ImportFrom) and node.level == 0 and node.module:
                names.add(node.module.split(".")[0])
        return names
    for path in glob.glob(os.path.join(root, "paper_2412_18106_amd", "*.py")):
        assert "oracle" not in imported(path), path
    for path in glob.glob(os.path.join(root, "oracle", "*.py")):
        assert "paper_2412_18106_amd" not in imported(path), path
    for name, allowed in (("bench.py", {"cpu_baseline"}), ("__graft_entry__.py", {"smoke"})):
        tree = ast.parse(open(os.path.join(root, name)).read())
        for fn in [n for n in ast.walk(tree) if isinstance(n, ast.FunctionDef)]:
            uses = any(isinstance(n, ast.ImportFrom) and n.module and n.module.split(".")[0] == "oracle"
                       for n in ast.walk(fn))
            assert not uses or fn.name in allowed, f"{name}: {fn.name} imports the oracle"
        top = [n for n in tree.body if isinstance(n, (ast.Import, ast.ImportFrom))]
        assert all("oracle" not in ast.dump(n) for n in top), name


def test_binding_refuses_to_import_without_the_library(tmp_path):
    """The product fails loudly when its library is missing: a copy of the package without libxyattn.so raises at
    import instead of falling back to anything."""
    import os
    import shutil
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    dst = tmp_path / "paper_2412_18106_amd"
    shutil.copytree(os.path.join(root, "paper_2412_18106_amd"), dst,
                    ignore=shutil.ignore_patterns("*.so", "*.so.sources", "__pycache__", "csrc"))
    res = subprocess.run([sys.executable, "-c", "import paper_2412_18106_amd.runner"], cwd=tmp_path,
                         capture_output=True, text=True, env={**os.environ, "PYTHONPATH": str(tmp_path)})
    assert res.returncode != 0 and "ImportError" in res.stderr and "no CPU fallback" in res.stderr
