"""The C-ABI library loads and exports every symbol include/step.h declares (no compute calls)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "step.h")
LIB = os.path.join(ROOT, "paper_2601_09093_amd", "libstep.so")


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    names = re.findall(r"^\s*(?:const\s+)?(?:int32_t|int|size_t|char\s*\*|void)\s*\*?\s*(\w+)\s*\(", src, flags=re.M)
    return sorted(set(names))


def test_header_declares_the_three_calls():
    names = declared_functions()
    for n in ("paged_decode_attn", "step_score", "prune_free", "step_attn_workspace_bytes",
              "step_score_workspace_bytes", "step_prune_workspace_bytes", "step_strerror", "step_version",
              "step_calib_copy", "step_profile_begin", "step_profile_end", "step_profile_kernel_name", "step_read_probe",
              "step_attn_waves_per_head", "step_attn_plan", "paged_decode_attn_planned",
              "step_reserve_workspace_bytes", "step_reserve_pages", "step_append_kv", "step_weighted_vote",
              "prune_free_static", "step_prune_static_max_pages", "step_freelist_rebuild", "step_freelist_add"):
        assert n in names, names


def test_library_exports_every_declared_symbol():
    if not os.path.exists(LIB):
        pytest.fail("libstep.so is not built: run python -m paper_2601_09093_amd.build")
    lib = ctypes.CDLL(LIB)
    for n in declared_functions():
        assert hasattr(lib, n), "missing export %s" % n


def test_host_only_entry_points():
    from paper_2601_09093_amd import binding
    L = binding.lib()
    assert L.step_version().decode() == "0.1"
    assert b"STEP_EPAGE" in L.step_strerror(16)
    d = binding.AttnDims(64, 32, 8, 128, 16, 2112, 100000, 0.088)
    assert binding.attn_workspace_bytes(d) > 64 * 32 * 130 * 4
    assert binding.attn_workspace_bytes(binding.AttnDims(4, 4, 1, 96, 16, 20, 10, 0.1)) == 0      # D unsupported
    assert binding.attn_workspace_bytes(binding.AttnDims(4, 4, 1, 64, 32, 20, 10, 0.1)) == 0      # P != 16
    assert binding.score_workspace_bytes(binding.ScoreDims(8, 256, 64, 8, 4, 1)) >= 4 * 8 * 4
    assert binding.score_workspace_bytes(binding.ScoreDims(8, 250, 64, 8, 4, 1)) == 0             # d % 128
    assert binding.prune_workspace_bytes(256, 1024, 150000) >= 256 + 150000 // 8


def test_binding_refuses_cpu_tensors():
    import torch
    from paper_2601_09093_amd import binding
    q = torch.zeros(1, 4, 64, dtype=torch.bfloat16)
    kp = torch.zeros(2, 1, 16, 64, dtype=torch.bfloat16)
    with pytest.raises(TypeError):
        binding.paged_decode_attn(q, kp, kp, torch.zeros(1, 2, dtype=torch.int32), torch.ones(1, dtype=torch.int32),
                                  out=q.clone(), workspace=torch.zeros(4096, dtype=torch.uint8))
