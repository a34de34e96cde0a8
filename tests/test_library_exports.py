"""The C-ABI library loads without a GPU and exports every function include/gear.h declares."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "gear.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gear_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_three_named_calls():
    names = declared_functions()
    for required in ("gear_init_tables", "gear_step", "gear_refresh_dfv"):
        assert required in names


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(os.path.join(ROOT, "paper_1806_03925_amd", "libgear.so"))
    for name in declared_functions():
        assert hasattr(lib, name), f"libgear.so does not export {name}"


def test_binding_mirrors_the_header():
    import paper_1806_03925_amd as g
    from paper_1806_03925_amd import binding
    assert sorted(binding.EXPORTS) == declared_functions()
    for name in binding.EXPORTS:
        assert hasattr(binding.lib, name)
    # host-only calls work without a GPU
    cfg = g.make_config(1000, 4096, 2000, 16, 64, (64, 1), max_batch=512, max_nnz=2048)
    assert g.gear_workspace_bytes(cfg) > 0
    assert g.gear_mlp_param_count(cfg) == 96 * 64 + 64 + 64 + 1
    assert g.gear_mlp_param_offset(cfg, 1, 0) == 96 * 64 + 64
    bad = g.make_config(1000, 4096, 2000, 12, 64, (64, 1), max_batch=512, max_nnz=2048)   # emb_dim % 8 != 0
    assert g.gear_workspace_bytes(bad) == 0 and g.gear_mlp_param_count(bad) == -1
    assert binding.lib.gear_status_string(3) == b"workspace or ready list too small"
    # null arguments are reported, not dereferenced
    assert binding.lib.gear_step(None, None, None, None, None, None, 1, 0.1, None, 0, None, None) == g.GEAR_ERR_INVALID
