"""The inline-assembly includes are committed so that the library builds without running their
generators; they must be exactly what the generators write (host only, no GPU)."""
import importlib.util
import os

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2510_14891_amd", "csrc")


def _load(name):
    spec = importlib.util.spec_from_file_location(name, os.path.join(CSRC, name + ".py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


@pytest.mark.parametrize("gen,inc", [("gen_pipe", "mttkrp_pipe.inc"), ("gen_rows_pipe", "mttkrp_rows_pipe.inc")])
def test_committed_include_matches_its_generator(gen, inc, tmp_path, monkeypatch, capsys):
    for var in ("MTTKRP_GEN_DEPTH", "MTTKRP_GEN_DEPTH_MIN", "MTTKRP_GEN_ONLY", "MTTKRP_GEN_ROWS_DEPTH",
                "MTTKRP_GEN_ROWS_XFLAGS"):
        monkeypatch.delenv(var, raising=False)
    out = str(tmp_path / inc)
    _load(gen).main(out)
    capsys.readouterr()
    with open(out) as f, open(os.path.join(CSRC, inc)) as g:
        assert f.read() == g.read(), "run paper_2510_14891_amd/build.py (or the generator) and commit the include"


def test_ring_registers_stay_inside_the_budget():
    """Every generated run keeps its ring inside the wavefront's register budget, leaves the
    accumulators and the allowance for the rest of the kernel below it, starts register tuples
    on even registers, and never asks for more outstanding loads than the counter can name."""
    for gen in ("gen_pipe", "gen_rows_pipe"):
        mod = _load(gen)
        tiles = getattr(mod, "TILES", [(a, b) for a in (1, 2, 3, 4) for b in (1, 2, 3, 4)])
        for w in (2, 1):
            for a, b in tiles:
                inst = mod.Inst(w, a, b)
                if not inst.budget:
                    continue
                assert inst.last_reg() < inst.budget <= 256, (gen, w, a, b)
                assert inst.t0 % 2 == 0 and inst.set % 2 == 0, (gen, w, a, b)
                assert inst.t0 >= inst.acc + mod.OTHERS[w], (gen, w, a, b)
                assert inst.d * inst.loads <= 63, (gen, w, a, b)
