"""CPU-only checks of the boundary: the library loads and exports every symbol the header declares."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "smoe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(smoe_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    import paper_2403_08245_amd as m
    names = _declared_symbols()
    assert len(names) >= 16
    for n in names:
        assert hasattr(m.lib, n), f"{n} declared in include/smoe.h but not exported by libsmoe.so"
    assert sorted(m.EXPORTS) == names


def test_host_side_argument_errors_need_no_gpu():
    import paper_2403_08245_amd as m
    assert m.lib.smoe_abi_version() == 1
    assert m.lib.smoe_strerror(0) == b"ok"
    assert b"invalid" in m.lib.smoe_strerror(-1)
    # a null context is rejected before any HIP call
    assert m.lib.smoe_topk_gate(None, None, None, 4, 4, 2, None, None) == -1
    assert m.lib.smoe_route(None, None, None, 4, 2, 4, None, None, None, None, 0) == -1
    assert m.lib.smoe_route_workspace_bytes(16384, 2, 8) >= 32 * 8 * 4
    assert m.lib.smoe_mlp_bwd_workspace_bytes(1, 2, 16, 2, 64, 32) > 0


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2403_08245_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src, f"{f} mentions the oracle"
