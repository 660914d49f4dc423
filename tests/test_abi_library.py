"""CPU-side checks of the C ABI library: it is built, loads, and exports every function include/bagpipe.h
declares; argument checks that need no GPU return the documented errors."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "bagpipe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bp_[a-z_0-9]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    import paper_2202_12429_amd as bp
    if not os.path.exists(bp.library_path()):
        from paper_2202_12429_amd.build import build
        build(verbose=False)
    return bp.load_library()


def test_header_declares_the_four_operations():
    names = declared_functions()
    for n in ("bp_oracle_plan", "bp_cache_apply", "bp_embbag_fwd", "bp_embbag_bwd_update"):
        assert n in names


def test_library_exports_every_declared_symbol(lib):
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} is declared in bagpipe.h but not exported"


def test_binding_has_the_same_names():
    import paper_2202_12429_amd as bp
    for n in ("bp_oracle_plan", "bp_cache_apply", "bp_embbag_fwd", "bp_embbag_bwd_update",
              "bp_oracle_plan_workspace_bytes", "bp_embbag_bwd_update_workspace_bytes"):
        assert callable(getattr(bp, n))


def test_config_struct_layout_matches_header():
    import paper_2202_12429_amd as bp
    assert ctypes.sizeof(bp.bp_config) == 64
    assert bp.bp_config.lookahead.offset == 28 and bp.bp_config.lr.offset == 32 and bp.bp_config.reserve.offset == 40
    assert bp.bp_config.cache_w_stride.offset == 48 and bp.bp_config.cache_state_stride.offset == 56


def test_argument_errors_without_gpu(lib):
    import paper_2202_12429_amd as bp
    assert bp.bp_version() >= 100
    assert "capacity" in bp.bp_error_string(-2)
    good = bp.make_config(1000, 64, 16)
    assert bp.bp_oracle_plan_workspace_bytes(good, 4096, 10) > 0
    assert bp.bp_embbag_bwd_update_workspace_bytes(good, 4096, 4096) > 0
    for bad in (bp.make_config(1000, 64, 6),              # 24-byte rows: not a multiple of 16 bytes
                bp.make_config(1000, 0, 16),               # no capacity
                bp.make_config(0, 64, 16),                 # no rows
                bp.make_config(1000, 64, 16, lookahead=-1),
                bp.make_config(1000, 64, 16, reserve=64),  # nothing left to plan with
                bp.make_config(1000, 64, 16, reserve=-1)):
        with pytest.raises(bp.BagpipeError) as e:
            bp.bp_embbag_bwd_update_workspace_bytes(bad, 128, 128)
        assert e.value.status == -1
    with pytest.raises(bp.BagpipeError) as e:
        bp.bp_embbag_bwd_update_workspace_bytes(bp.make_config(1000, 64, 512), 128, 128)   # 2 KiB rows
    assert e.value.status == -6
    with pytest.raises(bp.BagpipeError) as e:
        bp.bp_oracle_plan_workspace_bytes(good, 4096, 10_000)                               # too many batches
    assert e.value.status == -6
    # bf16 rows need dim % 8 == 0
    with pytest.raises(bp.BagpipeError):
        bp.bp_embbag_bwd_update_workspace_bytes(bp.make_config(1000, 64, 12, "bf16"), 128, 128)
