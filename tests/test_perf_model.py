"""Pins the reporting arithmetic to numbers the paper prints (Sec. IV-B)."""
import os

from paper_2510_14891_amd import perf_model as pm

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_table_model.txt")


def load():
    peak, shape, model, gf = {}, {}, [], []
    for line in open(GOLDEN):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] == "peak":
            peak[t[1]] = (float(t[2]) * 1e12, float(t[3]) * 1024.0 ** 4)
        elif t[0] == "shape":
            shape[t[1]] = tuple(int(v) for v in t[2:])
        elif t[0] == "model":
            model.append((t[1], t[2], float(t[3]), float(t[4])))
        elif t[0] == "gflops_check":
            gf.append((t[1], int(t[2]), float(t[3])))
    return peak, shape, model, gf


def test_predicted_times_match_table_model():
    peak, shape, model, _ = load()
    R = 32
    for tensor, dev, t_inf, t_0 in model:
        dims = shape[tensor]
        tau_f, tau_m = peak[dev]
        f = pm.flops_paper(dims, R)
        got_inf = pm.predicted_time(f, pm.m_inf(dims, R, 8), tau_f, tau_m)
        assert abs(got_inf - t_inf) <= 0.0015, (tensor, dev, got_inf, t_inf)
        # ELEM: N_T = 1, so the output term is N R whatever the mode
        got_0 = pm.predicted_time(f, pm.m_0(dims, R, 8, 0, 1), tau_f, tau_m)
        assert abs(got_0 - t_0) <= 0.015 * t_0, (tensor, dev, got_0, t_0)


def test_gflops_convention():
    _, shape, _, gf = load()
    for tensor, R, want in gf:
        f = pm.flops_paper(shape[tensor], R)
        assert abs(f / 1024.0 ** 3 - want) < 0.01
        # Table "width" best CUDA figure and Table "model" time agree through it
        assert abs(pm.gflops_paper_units(f, 0.0435) - 1328.3) < 2.0


def test_byte_models_order():
    dims, R = (401, 201, 12, 501), 32
    assert pm.m_inf(dims, R, 8) < pm.m_0_lm(dims, R, 8, 0, 216, 10) < pm.m_0(dims, R, 8, 0, 216)
    assert pm.flops_executed(dims, R) * len(dims) == 2 * pm.flops_paper(dims, R)
