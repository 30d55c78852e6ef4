"""The C-ABI library loads and exports every symbol include/rstitch.h declares;
host-side argument checks that need no GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    """Every function declared in include/*.h."""
    names = set()
    inc = os.path.join(ROOT, "include")
    for fn in sorted(os.listdir(inc)):
        if not fn.endswith(".h"):
            continue
        text = open(os.path.join(inc, fn)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names.update(re.findall(r"\b(rs_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_header_declares_the_four_calls():
    names = declared_functions()
    for n in ("rs_create_model", "rs_decode_step", "rs_catchup_prefill", "rs_route"):
        assert n in names


def test_library_exports_every_declared_symbol():
    import paper_2507_17307_amd as P
    lib = ctypes.CDLL(P.library_path())
    for n in declared_functions():
        assert hasattr(lib, n), n


def test_config_validation_on_the_host():
    import paper_2507_17307_amd as P
    import workloads as W
    ok = P.binding.make_config(W.S15, 4608)
    assert P.rs_workspace_bytes(ok) > 0
    assert P.rs_kv_bytes(ok) == 28 * 1 * 2 * 4608 * 128 * 2
    for field, value, word in [("max_seqs", 129, "max_seqs"), ("max_rows", 129, "max_rows"), ("head_dim", 48, "head_dim"),
                               ("n_kv_heads", 5, "divide"), ("vocab", 1, "vocab"), ("d_model", 1000, "multiples")]:
        cfg = P.binding.make_config(W.S15, 4608)
        setattr(cfg, field, value)
        assert P.rs_workspace_bytes(cfg) == 0 and word in P.rs_last_error()
    assert P.rs_route_scratch_bytes(0, 100) == 0 and P.rs_route_scratch_bytes(4, 1) == 0
    assert P.rs_route_scratch_bytes(4, 152064) > 0


def test_null_and_range_arguments_are_rejected_before_any_launch():
    import paper_2507_17307_amd as P
    lib = P.lib
    assert lib.rs_decode_step(None, 1, None, None, None, None, 0.5, 0, None, None, None) == -1
    assert lib.rs_catchup_prefill(None, 1, 1, None, None, None, None, None, 0.5, 0, None, None, None) == -1
    assert lib.rs_route(None, 1, 100, None, 0.5, 0, None, None, 0, None) == -1
    assert "null" in P.rs_last_error()
    assert lib.rs_stitch_generate(None, None, 0, None, 1, 1, 0, 0, None, 0.5, -1, None, 1, None, None) == -1
    assert lib.rs_route(16, 0, 100, None, 0.5, 0, 16, 16, 1 << 20, None) == -1
    assert lib.rs_route(16, 1, 1, None, 0.5, 0, 16, 16, 1 << 20, None) == -1
    assert lib.rs_route(16, 1, 100, None, 0.5, 7, 16, 16, 1 << 20, None) == -1
    assert lib.rs_route(16, 4, 152064, None, 0.5, 0, 16, 16, 64, None) == -1 and "scratch" in P.rs_last_error()
    out = ctypes.c_void_p()
    assert lib.rs_create_model(None, None, None, None, None, 0, ctypes.byref(out)) == -1
