"""Pins for oracle/overlap_model.py: the numbers the paper prints (App. C worked examples,
Table 1/2) and the limits it states (Sec. 3.3), none of which come from the oracle itself."""
import json
import os

import pytest

from oracle import overlap_model as om

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "overlap_examples.json")))


def _plat():
    p = GOLD["platform"]
    return om.Platform(p["p_peak_tflops"] * 1e12, p["bw_h2d_gbs"] * 1e9, p["eta_comp"], p["eta_pref"])


@pytest.mark.parametrize("model", ["wan", "flux", "hunyuan"])
def test_critical_configurations_app_c(model):
    m = GOLD["models"][model]
    plat = _plat()
    if model == "wan":
        g = lambda n: om.flops_dit(1, m["tokens_per_frame_unit"] * (n + m["frame_offset"]), m["d"], m["f"], m["l_ctx"])
    elif model == "flux":
        g = lambda b: om.flops_mmdit_avg(b, m["S"], m["d"], m["f"], m["l_ctx"], m["n_double"], m["n_single"])
    else:
        g = lambda n: om.flops_mmdit_avg(1, m["tokens_per_frame_unit"] * (n + m["frame_offset"]), m["d"], m["f"],
                                         m["l_ctx"], m["n_double"], m["n_single"])
    z = om.critical_config(g, m["b_pref_mb"] * 1e6, plat, GOLD["sp_degree"])
    assert abs(z - m["critical"]) <= GOLD["critical_tolerance"], z


def test_critical_needs_the_sp_share():
    # dropping the division by the SP degree lands far from the printed value: the pin bites
    m = GOLD["models"]["wan"]
    g = lambda n: om.flops_dit(1, 220 * (n + 3), m["d"], m["f"], m["l_ctx"])
    z = om.critical_config(g, 520e6, _plat(), 1)
    assert abs(z - 119.2) > 10


def test_parameter_bytes_app_b():
    assert om.bytes_single(3072, 12288) == 283_115_520
    assert om.bytes_double(3072, 12288) == 679_477_248
    # 7d^2+2df = modulation 3d^2 + lin1 (3d+f)d + lin2 (d+f)d
    d, f = 3072, 12288
    assert om.bytes_single(d, f) == 2 * (3 * d * d + (3 * d + f) * d + (d + f) * d)


def test_ridge_and_chunk_time():
    plat = _plat()
    assert om.i_star(plat) == pytest.approx(0.6 * 756e12 / (0.89 * 31.5e9))
    assert om.i_star(plat) == pytest.approx(16180, rel=1e-3)
    assert om.f_star(520e6, plat) / 520e6 == pytest.approx(om.i_star(plat))
    assert om.t_chunk(16e6, plat) * 1e3 == pytest.approx(0.571, abs=1e-3)


def test_hide_condition_and_residency_limits():
    plat = _plat()
    b = 520e6
    fs = om.f_star(b, plat)
    assert om.hidden(fs * 1.001, b, plat) and not om.hidden(fs * 0.999, b, plat)
    assert om.t_pref(b, plat, 1.0) == 0.0                       # 100 % residency: nothing to prefetch
    assert om.t_pref(b, plat, 0.0) == pytest.approx(b / (0.89 * 31.5e9))
    assert om.hidden(1.0, b, plat, resident_fraction=1.0)
    tc = om.t_comp(0.3 * fs, plat)
    prev_t, prev_m = None, None
    for r in (0, 0.2, 0.4, 0.6, 0.8, 1.0):
        t = om.step_time(tc, b, 30, plat, r)
        mem = om.weight_memory(b, 30, r)
        if prev_t is not None:
            assert t <= prev_t and mem >= prev_m                # Sec. 4.5: opposed monotone trends
        prev_t, prev_m = t, mem
    assert om.step_time(tc, b, 30, plat, 1.0) == pytest.approx(30 * tc)
    assert om.weight_memory(b, 30, 1.0) == pytest.approx(30 * b)
    assert om.weight_memory(b, 30, 0.0) == pytest.approx(2 * b)  # two layers live (Sec. 2.2)
    assert om.exposed_time(tc, b, 30, plat, 0.0) == pytest.approx(30 * (om.t_pref(b, plat) - tc))


def test_flop_formulas_scale_as_stated():
    # linear in B; quadratic in S only through attention (Sec. 3.1)
    d, f, L = 3072, 14336, 512
    assert om.flops_dit(2, 1000, d, f, L) == 2 * om.flops_dit(1, 1000, d, f, L)
    lin = lambda S: om.flops_dit(1, S, d, f, L) - 4 * S * S * d
    assert lin(2000) - lin(1000) == lin(3000) - lin(2000)
