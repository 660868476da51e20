"""Host-side checks of the C ABI (no GPU): exported symbols, layouts, error codes."""
import ctypes as C
import os
import re

import pytest

import paper_2211_00235_amd as pe
from oracle.params import param_table as oracle_table
from pe_inputs import CONFIGS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(os.path.join(ROOT, "paper_2211_00235_amd", "libpe_mi355x.so")):
        from paper_2211_00235_amd import build
        build.build()
    return pe.lib()


def test_every_declared_symbol_is_exported(L):
    hdr = open(os.path.join(ROOT, "include", "pe.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(pe_[a-z_]+)\s*\(", hdr))
    assert {"pe_block_fwd", "pe_block_bwd", "pe_stack_fwd_bwd", "pe_create"} <= names
    for n in sorted(names):
        assert hasattr(L, n), n


@pytest.mark.parametrize("name", list(CONFIGS))
def test_param_table_matches_oracle_layout(L, name):
    dims = dict(CONFIGS[name][0])
    ot, on = oracle_table(dims)
    assert pe.param_count(dims) == on
    lt = pe.param_table(dims)
    assert len(lt) == len(ot)
    for a, b in zip(lt, ot):
        assert a["name"] == b["name"] and a["offset"] == b["offset"]
        assert tuple(a["shape"]) == tuple(b["shape"]) and a["fan_in"] == b["fan_in"] and a["kind"] == b["kind"]


def test_dims_validation(L):
    d = dict(CONFIGS["af2_initial"][0])
    assert pe.check_dims(d) == 0
    for v in (1, 2):
        assert pe.check_dims(dict(d, variant=v)) == 0
    for key, bad in (("c_m", 250), ("d_msa", 64), ("dtype", 7), ("s", 0), ("c_z", 512), ("h_msa", 16), ("variant", 3),
                     ("variant", -1)):
        dd = dict(d)
        dd[key] = bad
        assert pe.check_dims(dd) == -2, key
        assert pe.workspace_bytes(dd, 1) == 0


def test_sizes_are_consistent(L):
    d = dict(CONFIGS["tiny"][0])
    assert pe.workspace_bytes(d, 1) >= pe.workspace_bytes(d, 0) + pe.ctx_bytes(d)
    tab = pe.ctx_table(d)
    assert all(e["offset_bytes"] % 256 == 0 for e in tab)
    end = max(e["offset_bytes"] + e["count"] * (2 if e["dtype"] == 1 else 4) for e in tab)
    assert end <= pe.ctx_bytes(d)
    assert pe.stack_workspace_bytes(0, None, 2, d) > pe.workspace_bytes(d, 1)
    # keeping every block's ctx: room for n ctx slots instead of one internal ctx
    keep = pe.stack_workspace_bytes(0, None, 3, d, keep=True)
    assert keep >= pe.stack_workspace_bytes(0, None, 3, d) + 2 * pe.ctx_bytes(d) - 4096
    # the orderings with the outer product mean in front save one more pair tensor (z0)
    assert pe.ctx_bytes(dict(d, variant=1)) > pe.ctx_bytes(d)
    assert pe.param_count(dict(d, variant=2)) == pe.param_count(d)


def test_null_and_error_strings(L):
    assert L.pe_block_fwd(None, None, None, None, None, None, None, None, None, None, None, 0, None, None) == -1
    assert L.pe_block_bwd(None, None, None, None, None, None, None, None, None, None, None, None, None, None, 0,
                          None, None) == -1
    assert L.pe_stack_workspace_bytes(0, None, 0, None) == 0
    for code in range(0, -7, -1):
        assert len(pe.strerror(code)) > 0
    assert pe.strerror(-3) == "workspace too small"


def test_dims_error_names_the_violated_limit(L):
    """Every limit that pe_check_dims enforces is reported in words (the header lists the same limits)."""
    d = dict(CONFIGS["af2_initial"][0])
    assert pe.dims_error(d) == ""
    for key, bad, word in (("c_m", 250, "multiples of 8"), ("d_msa", 64, "d_msa"), ("d_pair", 4, "d_pair"),
                           ("c_z", 512, "c_z must be <= 256"), ("c_tri", 200, "c_tri"), ("h_msa", 16, "h_msa"),
                           ("n_trans", 32, "n_trans"), ("variant", 3, "variant"), ("dtype", 7, "dtype"),
                           ("s", 0, "s and r")):
        dd = dict(d)
        dd[key] = bad
        assert pe.check_dims(dd) == -2, key
        assert word in pe.dims_error(dd), (key, pe.dims_error(dd))
    big = dict(d, s=70000, r=40000)          # s*r beyond the 32-bit row counts of the kernels
    assert pe.check_dims(big) == -2 and "2^31" in pe.dims_error(big)
    g = dict(CONFIGS["extra_msa"][0])
    assert pe.check_dims(dict(g, d_msa=16)) == -2 and "global column attention" in pe.dims_error(dict(g, d_msa=16))
    hdr = open(os.path.join(ROOT, "include", "pe.h")).read()
    for text in ("c_z <= 256", "c_tri <= 192", "n_trans*c_m <= 4096", "{8, 16, 24, 32}", "s*r < 2^31"):
        assert text in hdr, text


def test_static_scratch_size_is_exported(L):
    assert pe.static_scratch_bytes() == 32 << 20


def test_host_paths_under_sanitizers(tmp_path):
    """The host-only paths (dims validation, parameter and ctx tables, the dry-run plans behind every size query,
    argument validation of the compute calls) run in a build whose host code is instrumented with AddressSanitizer
    and UndefinedBehaviorSanitizer: tests/host_checks/abi_host_check.cpp walks them over the workload shapes,
    ragged and degenerate shapes and every limit of pe_dims; any report ends the program with a failure."""
    import subprocess
    from paper_2211_00235_amd import build
    exe = build.build_host_check(str(tmp_path / "abi_host_check"))
    res = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert res.stdout.startswith("ok "), res.stdout + res.stderr
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr, res.stderr
