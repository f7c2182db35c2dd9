"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2211_10017_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2211_10017_amd.build import build_library
        build_library()
    return binding.load()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "moe_wq.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert lib.moe_abi_version() == 4


def test_workspace_queries_are_host_functions(lib):
    assert lib.moe_permute_workspace_bytes(64, 2, 32) >= 16
    small = lib.moe_grouped_ffn_wq_workspace_bytes(128, 1024, 4096, 32, binding.MOE_F16)
    assert small >= 128 * 4096 * 2
    assert lib.moe_grouped_ffn_wq_workspace_bytes(128, 1024, 4096, 32, binding.MOE_BF16) > small
    assert lib.moe_permute_workspace_bytes(16384, 1, 64) >= 16 * 4 * 64 * 4


def test_bad_arguments_are_rejected_on_the_host(lib):
    vp = ctypes.c_void_p
    fake = vp(0x1000)          # never dereferenced: validation fails first
    assert lib.moe_quantize_experts(None, 1, 64, 32, 4, 0, None, None, None, None) == 1
    assert b"NULL" in lib.moe_last_error()
    assert lib.moe_quantize_experts(fake, 1, 64, 32, 3, 0, fake, fake, fake, None) == 2
    assert lib.moe_quantize_experts(fake, 1, 60, 32, 4, 0, fake, fake, fake, None) == 1
    assert lib.moe_quantize_experts(fake, 1, 128, 32, 4, 48, fake, fake, fake, None) == 1
    assert lib.moe_gate_topk(fake, 0, fake, None, None, 4, 64, 8, 3, 1, fake, fake, None) == 1      # k = 3
    assert lib.moe_gate_topk(fake, 0, fake, None, None, 4, 64, 1, 2, 1, fake, fake, None) == 1      # k > E
    assert lib.moe_gate_topk(fake, 2, fake, None, None, 4, 64, 8, 1, 1, fake, fake, None) == 2      # fp32 x
    assert lib.moe_gate_topk(fake, 0, fake, None, None, 4, 64, 300, 1, 1, fake, fake, None) == 2    # E too large
    assert lib.moe_permute(fake, fake, 0, 4, 1, 8, 60, fake, fake, fake, fake, None, 0, None) == 1   # row not 16 B
    assert lib.moe_permute(fake, fake, 0, 8192, 1, 8, 64, fake, fake, fake, fake, None, 0, None) == 3  # no workspace
    assert lib.moe_grouped_ffn_wq(fake, 0, fake, 8, 2, 0, 96, 128, 4, 0, 0, fake, fake, None, fake, fake, None,
                                  fake, 0, fake, 1 << 20, None) == 1                           # d % 64
    assert lib.moe_grouped_ffn_wq(fake, 0, fake, 8, 2, 0, 64, 128, 4, 0, 0, fake, fake, None, fake, fake, None,
                                  fake, 0, fake, 16, None) == 3                                # workspace too small
    assert b"workspace" in lib.moe_last_error()
    assert lib.moe_grouped_ffn_wq(fake, 0, fake, 8, 2, 0, 64, 128, 4, 0, 7, fake, fake, None, fake, fake, None,
                                  fake, 0, fake, 1 << 20, None) == 2                           # unknown activation
    assert lib.moe_combine(fake, 0, fake, fake, None, 4, 1, 60, fake, 2, None) == 1
    assert lib.moe_combine(fake, 5, fake, fake, None, 4, 1, 64, fake, 2, None) == 2


def test_fused_entry_points_say_on_the_host_what_they_take(lib):
    F16, BF16 = binding.MOE_F16, binding.MOE_BF16
    # routing fused into the tiled GEMMs: only sizes that run entirely in the tiled kernel, fp16 rows
    assert lib.moe_grouped_ffn_wq_routed_supported(16384, 64, 8192, 4096, 16384, 4, 128, F16) == 1
    assert lib.moe_grouped_ffn_wq_routed_supported(16384, 64, 8192, 4096, 16384, 4, 128, BF16) == 0
    assert lib.moe_grouped_ffn_wq_routed_supported(128, 32, 64, 1024, 4096, 4, 0, F16) == 0
    # a row bound of 64 alone does not mean streaming: 64 rows per expert are several row groups each, so row tiles
    assert lib.moe_grouped_ffn_wq_routed_supported(8192, 128, 64, 2048, 8192, 8, 0, F16) == 1
    assert lib.moe_grouped_ffn_wq_routed_supported(512, 128, 64, 2048, 8192, 8, 0, F16) == 0      # 4 rows per expert: one group, streams
    assert lib.moe_grouped_ffn_wq_routed_supported(256, 8, 256, 512, 2048, 8, 0, F16) == 0        # decode-sized: streams
    # permutation rebuilt inside fc1: decode sizes only; 2 = the un-permute may be fused in as well
    assert lib.moe_grouped_ffn_wq_gated_supported(64, 2, 32, 1024, 4096, 4, 0, F16) == 2        # the decode workload
    assert lib.moe_grouped_ffn_wq_gated_supported(256, 1, 8, 512, 2048, 8, 0, F16) == 2         # 256 assignments: the most
    assert lib.moe_grouped_ffn_wq_gated_supported(64, 2, 32, 1024, 8192, 4, 0, F16) == 1        # fc2's slabs too long to add into out
    assert lib.moe_grouped_ffn_wq_gated_supported(129, 2, 32, 1024, 4096, 4, 0, F16) == 0       # 258 assignments
    assert lib.moe_grouped_ffn_wq_gated_supported(64, 2, 32, 1024, 4096, 4, 128, F16) == 0      # group scales
    assert lib.moe_grouped_ffn_wq_gated_supported(64, 2, 32, 1024, 4096, 4, 0, BF16) == 0       # bf16 rows
    assert lib.moe_grouped_ffn_wq_gated_supported(64, 2, 32, 4096, 4096, 4, 0, F16) == 0        # fc1's slabs too long
    assert lib.moe_grouped_ffn_wq_gated_supported(64, 3, 32, 1024, 4096, 4, 0, F16) == 0        # k = 3
    vp = ctypes.c_void_p
    fake = vp(0x1000)          # never dereferenced: validation fails first
    gated = lib.moe_grouped_ffn_wq_gated
    assert gated(fake, 0, None, None, 64, 2, 32, 1024, 4096, 4, 0, 0, fake, fake, None, fake, fake, None, fake, 0,
                 fake, fake, fake, fake, 1 << 30, None) == 1                                     # no expert_idx
    assert gated(fake, 0, fake, None, 512, 1, 8, 1024, 4096, 4, 0, 0, fake, fake, None, fake, fake, None, fake, 0,
                 fake, fake, fake, fake, 1 << 30, None) == 2                                     # too many assignments
    assert b"decode-sized" in lib.moe_last_error()
    assert gated(fake, 0, fake, fake, 64, 2, 32, 1024, 4096, 4, 0, 0, fake, fake, None, fake, fake, None, fake, 0,
                 fake, fake, fake, fake, 1 << 30, None) == 2                                     # fused un-permute needs an fp32 output
    assert gated(fake, 0, fake, None, 64, 2, 32, 1024, 4096, 4, 0, 0, fake, fake, None, fake, fake, None, fake, 0,
                 fake, fake, fake, fake, 16, None) == 3                                          # workspace too small
    routed = lib.moe_grouped_ffn_wq_routed
    assert routed(fake, 0, fake, 2, fake, fake, 16384, 64, 8192, 4096, 16384, 4, 128, 0, fake, fake, None, fake, fake, None,
                  fake, 2, fake, 1 << 40, None) == 1                                             # fused un-permute needs k = 1
    assert routed(fake, 0, fake, 1, None, fake, 128, 32, 64, 1024, 4096, 4, 0, 0, fake, fake, None, fake, fake, None,
                  fake, 0, fake, 1 << 30, None) == 2                                             # decode sizes are not taken


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(binding.MoeError):
        binding.load()


def test_layer_level_limits_are_checked_before_anything_is_allocated(lib):
    """A whole layer call takes what its narrowest entry point takes: the gate's E <= 256 and k <= 2
    (moe_permute alone goes to 1024 experts and the FFN to 4096), and the FFN's d, F multiples of 64."""
    from paper_2211_10017_amd import MoEExpertLayer
    vp = ctypes.c_void_p
    fake = vp(0x1000)          # never dereferenced: validation fails first
    most = binding.LAYER_MAX_EXPERTS
    assert lib.moe_gate_topk(fake, 0, fake, None, None, 4, 64, most + 1, 1, 1, fake, fake, None) == 2
    assert b"above %d" % most in lib.moe_last_error()
    header = open(os.path.join(ROOT, "include", "moe_wq.h")).read()
    assert "k <= E <= %d" % most in header                      # the header's preamble states the same number
    for bad in (dict(E=most + 1, k=1), dict(E=8, k=3), dict(E=1, k=2), dict(E=8, k=0)):
        with pytest.raises(binding.MoeError, match="layer call"):
            MoEExpertLayer(16, 64, 128, bad["E"], bad["k"], 4, device="cpu")
    for d, F in ((96, 128), (64, 100), (0, 128)):
        with pytest.raises(binding.MoeError, match="multiples of 64"):
            MoEExpertLayer(16, d, F, 8, 1, 4, device="cpu")
