"""Host-side checks of the C ABI: the library loads and exports every declared symbol."""
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    names = set()
    for fn in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if fn.endswith(".h"):
            text = open(os.path.join(ROOT, "include", fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names |= set(re.findall(r"\b(flexmoe_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def _lib():
    from paper_2304_03946_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__ as g
        g.build()
    return binding, binding.load_library()


def test_header_declares_the_entry_points():
    assert set(_declared()) >= {"flexmoe_gate_topk", "flexmoe_route", "flexmoe_permute", "flexmoe_expert_ffn_fwd",
                                "flexmoe_expert_ffn_bwd", "flexmoe_combine", "flexmoe_workspace_bytes",
                                "flexmoe_status_str", "flexmoe_balance_ratio", "flexmoe_make_scheduling_plan",
                                "flexmoe_schedule", "flexmoe_placement_table"}


def test_library_exports_every_declared_symbol():
    binding, lib = _lib()
    for name in _declared():
        assert getattr(lib, name) is not None, name
    assert sorted(binding.EXPORTS) == _declared()


def test_status_strings_and_workspace_size():
    binding, lib = _lib()
    assert binding.status_str(binding.OK) == "ok"
    assert "placement" in binding.status_str(binding.BAD_PLACEMENT)
    # gpt_xl: workspace holds dHpre and act(Hpre), each A x f bf16, 256 fp32 partial tiles of 256 x 256 for
    # the split last round of the second forward product / dXp, and the work list of the weight gradients
    # (16 bytes per job and per slot of the 256-expert table, bucket offsets and K-tile count per expert, start and
    # rows per vExpert, the job count) and the table of 256-row tiles of the bucket list (16 bytes each, at most A / 256 + V of them, and a
    # header), each rounded up to 256 bytes
    ws = binding.flexmoe_workspace_bytes(65536, 2048, 8192, 64, 2, 96, binding.BF16)
    plan = (4 * 64 + 256) * 16 + (2 * 64 + 4 + 2 * 96) * 4      # one work list (with room for holes) and one length per weight-gradient product
    tiles = (131072 // 256 + 96 + 1) * 16
    assert ws == 2 * 131072 * 8192 * 2 + 256 * 256 * 256 * 4 + (plan + 255) // 256 * 256 + (tiles + 255) // 256 * 256
    assert binding.flexmoe_workspace_bytes(16, 12, 64, 4, 1, 4, binding.BF16) == 0      # d not a multiple of 8
    assert binding.flexmoe_workspace_bytes(16, 64, 64, 4, 5, 4, binding.BF16) == 0      # k > E


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2304_03946_amd")
    for fn in os.listdir(pkg):
        if fn.endswith(".py"):
            assert "oracle" not in open(os.path.join(pkg, fn)).read().replace("CPU oracle's tests", ""), fn


def test_argument_validation_needs_no_device():
    """Every entry point rejects bad arguments on the host, before any HIP call: these calls
    return a status here, on a machine without a GPU, and launch nothing."""
    import ctypes
    binding, lib = _lib()
    null = ctypes.c_void_p(None)
    one = ctypes.c_void_p(16)          # a non-null, 16-byte aligned address that is never dereferenced
    bf16, relu = binding.BF16, binding.RELU
    # dtype / activation outside the enums
    assert lib.flexmoe_gate_topk(one, one, 4, 64, 4, 1, 7, one, one, one, 1 << 20, null) == binding.UNSUPPORTED
    assert lib.flexmoe_expert_ffn_fwd(one, one, one, one, null, one, null, 4, 64, 64, 4, 4, 9, bf16, one, null, one, one,
                                      1 << 20, null) == binding.UNSUPPORTED
    # k > E, d not a multiple of 8, V < E
    assert lib.flexmoe_gate_topk(one, one, 4, 64, 4, 5, bf16, one, one, one, 1 << 20, null) == binding.INVALID_ARG
    assert lib.flexmoe_permute(one, one, null, 4, 1, 12, bf16, one, null) == binding.INVALID_ARG
    assert lib.flexmoe_combine(one, one, null, 4, 1, 12, bf16, one, null) == binding.INVALID_ARG
    assert lib.flexmoe_expert_ffn_bwd(one, one, one, null, one, one, one, one, 4, 64, 64, 4, 3, relu, bf16, one, one, one,
                                      one, 1 << 20, null) == binding.INVALID_ARG
    # null outputs
    assert lib.flexmoe_gate_bwd(one, one, one, one, one, one, one, one, one, one, 4, 64, 4, 2, 4, bf16, null, one,
                                one, one, 1 << 20, null) == binding.INVALID_ARG
    assert lib.flexmoe_gate_bwd(one, one, one, one, one, one, one, one, one, one, 4, 64, 4, 2, 4, bf16, one, one,
                                null, one, 1 << 20, null) == binding.INVALID_ARG
    # workspace too small
    assert lib.flexmoe_expert_ffn_fwd(one, one, one, one, null, one, null, 64, 64, 64, 4, 4, relu, bf16, one, one, one,
                                      one, 256, null) == binding.WORKSPACE_TOO_SMALL
    # a misaligned buffer for the kept activations
    assert lib.flexmoe_expert_ffn_fwd(one, one, one, one, null, one, null, 64, 64, 64, 4, 4, relu, bf16, one,
                                      ctypes.c_void_p(24), one, one, 1 << 20, null) == binding.INVALID_ARG
    assert lib.flexmoe_expert_bias_grads(one, one, one, 64, 64, 64, 4, 4, bf16, one, one, one, 256,
                                         null) == binding.WORKSPACE_TOO_SMALL
    assert lib.flexmoe_gate_bwd(one, one, one, one, one, one, one, one, one, one, 64, 64, 4, 2, 4, bf16, one, one,
                                one, one, 16, null) == binding.WORKSPACE_TOO_SMALL
    # the gathered forward exists for bf16 with d a multiple of 128 only
    assert lib.flexmoe_expert_ffn_fwd_gather(one, one, one, one, one, null, one, null, 64, 1, 64, 64, 4, 4, relu,
                                             bf16, one, null, one, one, 1 << 20, null) == binding.UNSUPPORTED
    assert lib.flexmoe_expert_ffn_fwd_gather(one, one, one, one, one, null, one, null, 64, 1, 128, 64, 4, 4, relu,
                                             binding.F32, one, null, one, one, 1 << 20, null) == binding.UNSUPPORTED
    # ... and addresses the gathered rows with 32-bit byte offsets below 2^31: N * d below 2^30
    assert lib.flexmoe_expert_ffn_fwd_gather(one, one, one, one, one, null, one, null, 1 << 22, 1, 256, 128, 4, 4, relu,
                                             bf16, one, null, one, one, 1 << 40, null) == binding.UNSUPPORTED
    # the top-1 forward needs d and f multiples of 128
    assert lib.flexmoe_expert_ffn_fwd_top1(one, one, one, one, one, null, one, null, 64, 128, 64, 4, 4, relu, bf16, one,
                                           null, one, one, 1 << 20, null) == binding.UNSUPPORTED
    assert lib.flexmoe_expert_ffn_fwd_top1(one, one, one, one, one, null, one, null, 64, 128, 128, 4, 4, relu, bf16, one,
                                           null, null, one, 1 << 20, null) == binding.INVALID_ARG
    assert lib.flexmoe_expert_ffn_bwd_top1(one, one, one, null, one, one, one, one, one, 64, 128, 64, 4, 4, relu, bf16, one,
                                           one, one, one, 1 << 20, null) == binding.UNSUPPORTED
    # a placement table that leaves an expert without a vExpert (host arrays: these are read)
    off = (ctypes.c_int32 * 3)(0, 2, 2)
    ids = (ctypes.c_int32 * 2)(0, 1)
    assert lib.flexmoe_route(one, 4, 1, 2, 2, off, ids, one, one, one, one, one, one, one, 1 << 20,
                             null) == binding.BAD_PLACEMENT
