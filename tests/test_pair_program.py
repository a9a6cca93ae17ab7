"""Host logic of the paired enumeration kernel: the jump tables its precompute step writes (csrc/ppo_pair_program.h,
compiled for the host) are walked through a model of the generated code; every walk must end and leave the window
minima of Sec. III-B's memory rule in the registers.  No GPU."""
import importlib.util
import os

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _checker():
    path = os.path.join(ROOT, "paper_2210_12219_amd", "csrc", "check_pair_program.py")
    spec = importlib.util.spec_from_file_location("check_pair_program", path)
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_tables_walk_to_the_end_and_give_window_minima():
    rows, jumps = _checker().run_checks(n_random=300, seed=11)
    assert rows > 2000 and jumps > rows


def test_a_wrong_table_is_caught():
    """the model refuses a jump into the middle of nowhere and a walk that does not end"""
    import numpy as np
    import pytest
    mod = _checker()
    model = mod.Model()
    entry = np.full(model.nslot, model.end, dtype=np.uint16)
    entry[(10 - 1) % model.nslot] = 3          # not the start of anything
    with pytest.raises(AssertionError):
        model.walk(entry, 10, [0] * (model.umax + 1))
    # a piece of run code whose header's entry sends the walk back to itself
    kind_run = [t for t, v in model.at.items() if v == ("run", 5, 6)][0]
    entry = np.full(model.nslot, model.end, dtype=np.uint16)
    entry[(10 - 1) % model.nslot] = kind_run
    entry[(6 - 1 - 1) % model.nslot] = kind_run
    with pytest.raises(AssertionError):
        model.walk(entry, 10, [0x0400] * (model.umax + 1))
