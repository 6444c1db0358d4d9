"""Pins of the saturation-threshold oracle (Eq. 1 and App. B.4 Eq. 3 of the paper) and the
library's host-side implementations of the same formulas (pure host arithmetic, no GPU)."""
import os

import pytest

import paper_2605_02960_amd as moe
from paper_2605_02960_amd import build as moe_build
from oracle import saturation as sat


@pytest.fixture(scope="module", autouse=True)
def _lib():
    moe_build.ensure_built()


def test_flops_per_token_of_the_qwen3_shaped_block():
    # 8 routed rows of 6*H*I = 37 748 736 flop each, plus the router's 2*H*E
    assert sat.flops_per_token(4096, 128, 8, 1536) == 8 * 37748736 + 2 * 4096 * 128 == 303038464.0
    cfg = moe.make_config(65536, 4096, 128, 8, 1536, moe.DTYPE_BF16, moe.DTYPE_BF16)
    assert moe.moe_layer_flops_per_token(cfg) == 303038464.0


def test_eq1_is_time_times_rate_times_margin():
    # 4 ms of transfer on a 2.5 PFLOP/s part with the paper's example margin 1.2 -> 12 TFLOP
    assert sat.threshold_eq1(4e-3, 2.5e15, 1.2) == pytest.approx(1.2e13, rel=1e-15)
    assert sat.threshold_eq1(1.0, 1.0, 1.0) == 1.0
    assert sat.threshold_eq1(2e-3, 1e15) == 2 * sat.threshold_eq1(1e-3, 1e15)        # linear in t_EP
    assert sat.threshold_eq1(0.0, 1e15) == 0.0
    for args in ((4e-3, 2.5e15, 1.2), (0.09, 1.0e15, 1.0), (1e-3, 5e15, 1.5)):
        assert moe.moe_saturation_threshold_flops(*args) == sat.threshold_eq1(*args)


def test_eq3_special_cases_stated_by_the_paper():
    c = 3.0e14
    # transfers hidden: collapses to gamma * C_dummy
    assert sat.threshold_calibrated(10e-3, 8e-3, c, 1.2) == 1.2 * c
    assert sat.threshold_calibrated(10e-3, 10e-3, c, 1.2) == 1.2 * c
    # transfers exposed: the ratio t_e / t_c scales the reference batch
    assert sat.threshold_calibrated(10e-3, 25e-3, c, 1.2) == pytest.approx(1.2 * 2.5 * c, rel=1e-15)
    # the fallback before calibration equals Eq. 3 with t_e / t_c = 1
    f_tok, n_ref = sat.flops_per_token(4096, 128, 8, 1536), 65536
    assert sat.threshold_fallback(f_tok, n_ref, 1.2) == sat.threshold_calibrated(1.0, 1.0, f_tok * n_ref, 1.2)
    assert sat.threshold_calibrated(None, 5.0, c, 1.2) == 1.2 * c
    for args in ((10e-3, 8e-3, c, 1.2), (10e-3, 25e-3, c, 1.2), (0.0, 5.0, c, 1.2), (3e-3, 3e-3, c, 1.0)):
        assert moe.moe_calibrated_threshold_flops(*args) == sat.threshold_calibrated(*args)


def test_eq3_agrees_with_eq1_when_later_layers_are_transfer_bound():
    """If the later layers last exactly the transfer time (t_e = t_EP) and the reference batch runs at
    F = C_dummy / t_c flop/s, Eq. 3 is Eq. 1 at that rate."""
    t_ep, t_c, c = 88e-3, 21e-3, 65536 * sat.flops_per_token(4096, 128, 8, 1536)
    assert sat.threshold_calibrated(t_c, t_ep, c, 1.2) == pytest.approx(sat.threshold_eq1(t_ep, c / t_c, 1.2), rel=1e-14)


def test_delivery_and_fallback_rules():
    """App. B.4: a pinned value wins; before calibration T = gamma * f_tok * n_ref; without f_tok the
    same rule runs in tokens, and the two units differ exactly by the factor f_tok."""
    f_tok, n_ref = sat.flops_per_token(4096, 128, 8, 1536), 65536
    assert sat.resolve_threshold(7.5e15, 10e-3, 25e-3, f_tok, n_ref) == (7.5e15, "flops")       # pinned: no update
    assert sat.resolve_threshold(None, None, None, f_tok, n_ref, 1.2) == (sat.threshold_fallback(f_tok, n_ref, 1.2), "flops")
    assert sat.resolve_threshold(0.0, 10e-3, 25e-3, f_tok, n_ref, 1.2) == (sat.threshold_calibrated(10e-3, 25e-3, f_tok * n_ref, 1.2), "flops")
    t_tok, unit = sat.resolve_threshold(None, 10e-3, 25e-3, None, n_ref, 1.2)
    assert unit == "tokens" and t_tok == pytest.approx(1.2 * 2.5 * n_ref, rel=1e-15)
    t_fl, _ = sat.resolve_threshold(None, 10e-3, 25e-3, f_tok, n_ref, 1.2)
    assert t_fl == pytest.approx(t_tok * f_tok, rel=1e-15)
    assert sat.resolve_threshold(4096.0, 1.0, 9.0, 0.0, n_ref) == (4096.0, "tokens")
    # the library's host routine: same values, same unit
    units = {"flops": 0, "tokens": 1}
    for args in ((7.5e15, 10e-3, 25e-3, f_tok, n_ref, 1.2), (0.0, 0.0, 0.0, f_tok, n_ref, 1.2),
                 (0.0, 10e-3, 25e-3, f_tok, n_ref, 1.2), (0.0, 10e-3, 25e-3, 0.0, n_ref, 1.2),
                 (0.0, 10e-3, 5e-3, float("nan"), n_ref, 1.5), (4096.0, 1.0, 9.0, 0.0, n_ref, 1.2)):
        want_t, want_u = sat.resolve_threshold(args[0] or None, args[1] or None, args[2], None if not args[3] > 0 else args[3], *args[4:])
        assert moe.moe_resolve_threshold(*args) == (want_t, units[want_u]), args
    for bad in ((0.0, 1.0, 1.0, 1.0, 1.0, 0.0), (0.0, 1.0, 1.0, 1.0, -1.0, 1.2)):
        with pytest.raises(moe.MoEError) as e:
            moe.moe_resolve_threshold(*bad)
        assert e.value.status == -2
