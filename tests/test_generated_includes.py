"""The inline-assembly includes of the two kernels are build products of their generators
(written by build.py on every build).  The generators must be deterministic, and every run they
emit must fit the register budget it claims (host only, no GPU)."""
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
def test_generator_is_deterministic_and_matches_the_built_include(gen, inc, tmp_path, capsys):
    a, b = str(tmp_path / ("a_" + inc)), str(tmp_path / ("b_" + inc))
    _load(gen).main(a)
    _load(gen).main(b)
    capsys.readouterr()
    text = open(a).read()
    assert text == open(b).read()
    assert "asm volatile" in text and "s_waitcnt vmcnt(" in text
    built = os.path.join(CSRC, inc)
    if os.path.exists(built):       # the include the library in the tree was compiled from
        assert open(built).read() == text, "stale include: run python -m paper_2510_14891_amd.build"


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
