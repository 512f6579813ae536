"""The C-ABI shared library: builds for gfx950, loads, exports every function the
header declares, and rejects bad arguments on the host (no GPU work here)."""
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2506_15050_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build()
    return binding.load()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "tppo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tppo_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound(lib):
    from paper_2506_15050_amd import binding
    names = _declared_functions()
    assert "tppo_token_logprobs" in names and "tppo_egae" in names and "tppo_ppo_losses" in names
    assert "tppo_select" in names
    for n in names:
        assert getattr(lib, n) is not None
    assert sorted(binding.EXPORTS) == names
    assert lib.tppo_version() >= 100


def test_workspace_queries(lib):
    assert lib.tppo_token_logprobs_workspace_bytes(0, 64, 1000, 1) >= 256
    big = lib.tppo_token_logprobs_workspace_bytes(88600, 5120, 152064, 1)
    assert 3 * 4 * 88600 <= big <= 3 * 4 * 88600 * 64 + 256
    assert lib.tppo_egae_workspace_bytes(2_400_000, 512) >= 2_400_000 // 1024 * 48
    assert lib.tppo_ppo_losses_workspace_bytes(10, 1) >= 32
    assert lib.tppo_plan_bytes(2_400_000, 512) == lib.tppo_egae_workspace_bytes(2_400_000, 512)


def test_host_side_argument_errors(lib):
    N, S, P, D, W = -1, -2, -3, -4, -5
    # egae: parameter range, sizes, NULLs, workspace -- all detected before any launch
    assert lib.tppo_egae(None, None, None, None, None, 1, 10, 1.5, 0.5, None, None, None, 0, None, None, None) == P
    assert lib.tppo_egae(None, None, None, None, None, 1, 10, 1.0, -0.1, None, None, None, 0, None, None, None) == P
    assert lib.tppo_egae(None, None, None, None, None, 1, -1, 1.0, 0.5, None, None, None, 0, None, None, None) == S
    assert lib.tppo_egae(None, None, None, None, None, 1, 10, 1.0, 0.5, None, None, None, 0, None, None, None) == N
    assert lib.tppo_egae(None, None, None, None, None, 0, 0, 1.0, 0.5, None, None, None, 0, None, None, None) == 0
    assert lib.tppo_egae(256, 256, 256, 256, None, 1, 10, 1.0, 0.5, 256, 256, None, 0, None, None, None) == W
    assert lib.tppo_egae(256, 256, 256, 256, None, 1, 10, 1.0, 0.5, 256, 256, 128, 1 << 20, None, None, None) == W  # misaligned
    # select
    assert lib.tppo_select(None, None, None, None, 1, 1, 0, None, None, None, None, None, None, 0, None, None, 0, None, 0, None, None) == N
    assert lib.tppo_select(256, 256, 256, None, 1, 1, -1, 256, 256, 256, None, None, None, 0, 256, None, 0, None, 0, None, None) == P
    assert lib.tppo_select(256, 256, 256, None, -1, 1, 0, 256, 256, 256, None, None, None, 0, 256, None, 0, None, 0, None, None) == S
    assert lib.tppo_select(256, 256, 256, None, 1, 1, 0, 256, 256, 256, None, 256, None, 4, 256, None, 0, None, 0, None, None) == N  # targets without ids
    assert lib.tppo_select(256, 256, 256, None, 1, 1, 0, 256, 256, 256, 256, None, None, 4, 256, None, 0, None, 0, None, None) == W  # indices need a workspace
    assert lib.tppo_select(256, 256, 256, None, 1, 1, 0, 256, 256, 256, None, None, None, 0, 256, None, 0, 256, 16, None, None) == W  # plan too small
    assert lib.tppo_select(256, 256, 256, None, 1, 1, 0, 256, 256, 256, None, None, None, 0, 256, None, 0, 264, 1 << 20, None, None) == W  # plan misaligned
    # plan
    assert lib.tppo_plan_build(None, None, None, 1, 4, 256, 1 << 20, None, None) == N
    assert lib.tppo_plan_build(256, None, 256, 1, -4, 256, 1 << 20, None, None) == S
    assert lib.tppo_plan_build(256, None, 256, 1, 4, 256, 16, None, None) == W
    assert lib.tppo_plan_build(256, None, 256, 1, 4, None, 1 << 20, None, None) == W
    assert lib.tppo_egae(256, 256, 256, 256, None, 1, 10, 1.0, 0.5, 256, 256, None, 0, 264, None, None) == W       # plan misaligned
    # token_logprobs
    assert lib.tppo_token_logprobs(256, 4, 64, 64, 256, 100, 64, 7, 256, 256, 4, None, None, 256, None, None, 0, None, None) == D
    assert lib.tppo_token_logprobs(256, 4, 64, 32, 256, 100, 64, 0, 256, 256, 4, None, None, 256, None, None, 0, None, None) == S  # ld < H
    assert lib.tppo_token_logprobs(256, 4, 64, 64, 256, 100, 64, 0, 256, 256, 0, None, None, 256, None, None, 0, None, None) == 0  # M = 0
    assert lib.tppo_token_logprobs(None, 4, 64, 64, 256, 100, 64, 0, 256, 256, 4, None, None, 256, None, None, 0, None, None) == N
    assert lib.tppo_token_logprobs(256, 4, 64, 64, 256, 100, 64, 1, 256, 256, 4, None, None, 256, None, None, 0, None, None) == W  # bf16 MFMA path needs workspace
    # losses
    assert lib.tppo_ppo_losses(None, None, None, None, None, None, 256, 256, 256, 1, 4, -0.1, 0.2, 0.5, 0.6, 256, 256, 1 << 20, None, None, None) == P
    assert lib.tppo_ppo_losses(256, None, 256, None, None, None, 256, 256, 256, 1, 4, 0.2, 0.2, 0.5, 0.6, 256, 256, 1 << 20, None, None, None) == N
    assert lib.tppo_ppo_losses(None, None, None, None, None, None, 256, 256, 256, 1, 4, 0.2, 0.2, 0.5, 0.6, None, 256, 1 << 20, None, None, None) == N
    assert lib.tppo_ppo_losses(None, None, None, None, None, None, 256, 256, 256, 1, 4, 0.2, 0.2, 0.5, 0.6, 256, None, 0, None, None, None) == W
    # loss derivatives: same checks, plus gradient pointers that must match their halves, and the scales
    bw = lib.tppo_ppo_losses_backward
    assert bw(256, 256, 256, None, None, None, 256, 256, 256, 1, 4, 0.2, 0.2, 0.5, 0.6, 1.0, 1.0, 0, 0, None, None, None, None, 256, 1 << 20, None, None, None) == N
    assert bw(256, 256, 256, None, None, None, 256, 256, 256, 1, 4, 0.2, 0.2, 0.5, 0.6, 1.0, 1.0, 0, 0, 256, 256, None, None, 256, 1 << 20, None, None, None) == N
    assert bw(256, 256, 256, None, None, None, 256, 256, 256, 1, 4, 0.2, -1.0, 0.5, 0.6, 1.0, 1.0, 0, 0, 256, None, None, None, 256, 1 << 20, None, None, None) == P
    assert bw(256, 256, 256, None, None, None, 256, 256, 256, 1, 4, 0.2, 0.2, 0.5, 0.6, float("nan"), 1.0, 0, 0, 256, None, None, None, 256, 1 << 20, None, None, None) == P
    assert bw(256, 256, 256, None, None, None, 256, 256, 256, 1, 4, 0.2, 0.2, 0.5, 0.6, 1.0, 1.0, 0, 0, 256, None, None, None, None, 0, None, None, None) == W
    assert bw(256, 256, 256, None, None, None, 256, 256, 256, 1, -4, 0.2, 0.2, 0.5, 0.6, 1.0, 1.0, 0, 0, 256, None, None, None, 256, 1 << 20, None, None, None) == S
    assert lib.tppo_ppo_losses_backward_workspace_bytes(10, 1) >= 5 * 8
    # value head
    vh = lib.tppo_value_head
    assert vh(256, 4, 64, 64, 256, 0.0, 0, None, None, 4, None, 256, None, None) == D          # fp32 not offered
    assert vh(256, 4, 60, 64, 256, 0.0, 1, None, None, 4, None, 256, None, None) == P          # H % 8
    assert vh(256, 4, 64, 32, 256, 0.0, 1, None, None, 4, None, 256, None, None) == S          # ld < H
    assert vh(256, 4, 64, 64, None, 0.0, 1, None, None, 4, None, 256, None, None) == N
    assert vh(256, 4, 64, 64, 256, 0.0, 1, None, None, 0, None, 256, None, None) == 0          # M = 0
    # diagnostic streams
    assert lib.tppo_diag_streams(None, None, 64, 64, 1, 0, None) == N
    assert lib.tppo_diag_streams(256, None, 40, 64, 1, 0, None) == S
    assert lib.tppo_diag_streams(264, None, 64, 64, 1, 0, None) == P
    assert lib.tppo_diag_streams(256, 512, 64, 64, 3, 3, None) == P              # not one of the offered shapes
    # diagnostic loop
    assert lib.tppo_diag_mfma_rate(None, None, 10, None, None) == N
    assert lib.tppo_diag_mfma_rate(256, 256, -1, None, None) == S
    assert lib.tppo_diag_mfma_rate(264, 256, 10, None, None) == P          # operands not 16-byte aligned


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    from paper_2506_15050_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        binding.load()
