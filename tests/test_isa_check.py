"""The build's check on the compiler's output for the hand-issued scalar loads (CPU only)."""
import pytest

from paper_2211_13878_amd import build
from paper_2211_13878_amd.isa_check import count_requests, scalar_prefetch_violations

GOOD = """
_Zkernel:                               ; @_Zkernel
\ts_load_dwordx8 s[20:27], s[0:1], 0x0  ; the compiler's own load: it waits before touching s[20:27]
\ts_cbranch_scc1 .LBB0_9
\t;;#ASMSTART
\ts_load_dwordx16 s[36:51], s[0:1], 0x0
\ts_load_dwordx16 s[52:67], s[0:1], 0x40
\t;;#ASMEND
\t;;#ASMSTART
\tv_add_f64 v[58:59], v[56:57], s[4:5]
\tv_min_f64 v[42:43], v[42:43], v[58:59]
\t;;#ASMEND
\ts_add_u32 s2, s2, 8                     ; unrelated scalar work is fine
\ts_nop 0
\ts_waitcnt lgkmcnt(0)
\tv_add_f64 v[58:59], v[56:57], s[36:37]
\ts_cbranch_scc1 .LBB0_1
"""


def test_clean_sequence_passes():
    assert scalar_prefetch_violations(GOOD) == [] and count_requests(GOOD) == 2


def test_spill_of_an_in_flight_register_is_caught():
    bad = GOOD.replace("\ts_nop 0\n", "\tv_writelane_b32 v53, s40, 7\n")
    v = scalar_prefetch_violations(bad)
    assert len(v) == 1 and v[0][0] == "_Zkernel" and "v_writelane_b32" in v[0][3]


def test_reuse_of_an_in_flight_register_pair_is_caught():
    bad = GOOD.replace("s_add_u32 s2, s2, 8 ", "s_lshl_b64 s[66:67], s[2:3], 3 ")
    assert len(scalar_prefetch_violations(bad)) == 1


def test_weaker_wait_does_not_count_and_control_flow_is_caught():
    # scalar loads return out of order: only lgkmcnt(0) guarantees arrival
    bad = GOOD.replace("s_waitcnt lgkmcnt(0)", "s_waitcnt lgkmcnt(1)")
    v = scalar_prefetch_violations(bad)
    assert v and all("s[36:37]" in x[3] or "control flow" in x[3] for x in v)
    bad = GOOD.replace("\ts_nop 0\n", "\ts_cbranch_vccz .LBB0_2\n")
    assert any("control flow" in x[3] for x in scalar_prefetch_violations(bad))
    bad = GOOD.replace("\ts_nop 0\n", ".LBB0_7:\n")
    assert any("label" in x[3] for x in scalar_prefetch_violations(bad))


def test_product_device_code_is_clean():
    """Compiles the kernels to gfx950 assembly with the library's flags and checks every request."""
    assert build.check_isa() >= 100        # every sweep variant x storage mode x back-pointer width


def test_library_in_tree_is_stamped_and_an_unstamped_one_is_refused(tmp_path, monkeypatch):
    """The build step stamps what it has checked; the binding loads nothing else."""
    import subprocess
    from paper_2211_13878_amd import binding
    assert binding.galv_dp_build_stamp().startswith("isa-checked ")
    assert build.compiler_id().split("|")[0].strip() in binding.galv_dp_build_stamp()
    # a library built by hand: same symbol, no stamp from the checked build
    src = tmp_path / "fake.c"
    src.write_text('const char *galv_dp_build_stamp(void) { return "unchecked"; }\n')
    lib = tmp_path / "libfake.so"
    subprocess.check_call(["gcc", "-shared", "-fPIC", "-o", str(lib), str(src)])
    monkeypatch.setattr(binding, "LIB_PATH", str(lib))
    monkeypatch.setattr(binding, "_lib", None)
    with pytest.raises(ImportError, match="unverified"):
        binding.load_library()
    # and one without the symbol at all
    src.write_text("int nothing_here(void) { return 0; }\n")
    lib = tmp_path / "libfake2.so"                      # a new name: the loader caches by path
    subprocess.check_call(["gcc", "-shared", "-fPIC", "-o", str(lib), str(src)])
    monkeypatch.setattr(binding, "LIB_PATH", str(lib))
    with pytest.raises(ImportError, match="no stamp"):
        binding.load_library()


def test_build_has_no_way_around_the_check():
    import inspect
    assert "check" not in inspect.signature(build.build_library).parameters
