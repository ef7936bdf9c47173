"""Host-side checks of the planner hook: the reward metric of Section 4.3
(RW = SM * FLT, MPS = RW / (PC + RC)), the compress-or-recompute branch of Algorithm 1, and
that the saved-tensor hooks leave ineligible tensors alone (CPU tensors here, so no kernel
runs)."""
from __future__ import annotations

from fractions import Fraction

import pytest

torch = pytest.importorskip("torch")

from paper_2510_11400_amd import hooks


def test_mps_is_saved_memory_times_freed_lifetime_over_purge_plus_regain_cost():
    # exact rational arithmetic on values that are exact in binary64
    sm, flt, pc, rc = 3 * 2 ** 20, 0.5, 0.125, 0.375
    assert hooks.mps(sm, flt, pc, rc) == float(Fraction(sm) * Fraction(flt) / (Fraction(pc) + Fraction(rc)))
    assert hooks.mps(sm, flt, pc, rc) == 3 * 2 ** 20            # 0.5 / 0.5 = 1
    # doubling the lifetime doubles the reward; doubling both costs halves it; no saving, no reward
    assert hooks.mps(sm, 2 * flt, pc, rc) == 2 * hooks.mps(sm, flt, pc, rc)
    assert hooks.mps(sm, flt, 2 * pc, 2 * rc) == hooks.mps(sm, flt, pc, rc) / 2
    assert hooks.mps(0, flt, pc, rc) == 0
    with pytest.raises(ValueError):
        hooks.mps(sm, flt, 0.0, 0.0)


def test_the_plan_evicts_only_when_recomputation_rewards_more():
    assert hooks.prefer_recompute(2.0, 1.0) is True
    assert hooks.prefer_recompute(1.0, 2.0) is False
    assert hooks.prefer_recompute(1.0, 1.0) is False            # a tie compresses (the else branch)


def test_hooks_pass_ineligible_tensors_through_untouched():
    x = torch.randn(64, 128, requires_grad=True)               # CPU: not eligible
    w = torch.nn.Parameter(torch.randn(32, 128))
    ctx = hooks.SavedActivations(min_numel=1, record=True)
    with ctx:
        y = torch.nn.functional.relu(x @ w.t()).sum()
    y.backward()
    ref_x = torch.randn(0)
    x2 = x.detach().clone().requires_grad_(True)
    w2 = torch.nn.Parameter(w.detach().clone())
    torch.nn.functional.relu(x2 @ w2.t()).sum().backward()
    assert torch.equal(x.grad, x2.grad) and torch.equal(w.grad, w2.grad)
    assert ctx.records == [] and ctx.next_tensor_id == 0 and ref_x.numel() == 0
