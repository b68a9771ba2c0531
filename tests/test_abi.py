"""Host-side checks of the C ABI: the library loads and exports every declared symbol."""
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "flexmoe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(flexmoe_[a-z0-9_]+)\s*\(", text)))


def _lib():
    from paper_2304_03946_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__ as g
        g.build()
    return binding, binding.load_library()


def test_header_declares_the_entry_points():
    assert set(_declared()) >= {"flexmoe_gate_topk", "flexmoe_route", "flexmoe_permute", "flexmoe_expert_ffn_fwd",
                                "flexmoe_expert_ffn_bwd", "flexmoe_combine", "flexmoe_workspace_bytes",
                                "flexmoe_status_str"}


def test_library_exports_every_declared_symbol():
    binding, lib = _lib()
    for name in _declared():
        assert getattr(lib, name) is not None, name
    assert sorted(binding.EXPORTS) == _declared()


def test_status_strings_and_workspace_size():
    binding, lib = _lib()
    assert binding.status_str(binding.OK) == "ok"
    assert "placement" in binding.status_str(binding.BAD_PLACEMENT)
    # gpt_xl: workspace holds dHpre and act(Hpre), each A x f bf16
    ws = binding.flexmoe_workspace_bytes(65536, 2048, 8192, 64, 2, 96, binding.BF16)
    assert ws == 2 * 131072 * 8192 * 2
    assert binding.flexmoe_workspace_bytes(16, 12, 64, 4, 1, 4, binding.BF16) == 0      # d not a multiple of 8
    assert binding.flexmoe_workspace_bytes(16, 64, 64, 4, 5, 4, binding.BF16) == 0      # k > E


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2304_03946_amd")
    for fn in os.listdir(pkg):
        if fn.endswith(".py"):
            assert "oracle" not in open(os.path.join(pkg, fn)).read().replace("CPU oracle's tests", ""), fn
