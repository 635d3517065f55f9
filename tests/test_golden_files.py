"""The stored full-length oracle results under tests/golden/ belong to the oracle and the input
generators as they stand (a digest of their sources travels with every file), hold what the GPU
tests read, and were written by the committed script, which touches nothing but the oracle."""
import os

import numpy as np
import pytest

import workloads as WL
from gpu_util import golden_source_digest, load_golden

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_generator_calls_only_the_oracle():
    text = open(os.path.join(ROOT, "tests", "golden", "make_full_length_expectations.py")).read()
    assert "paper_2003_10735_amd" not in text and "import torch" not in text
    assert "import oracle as O" in text and "import workloads as WL" in text


@pytest.mark.parametrize("name", ["batch4", "clip"])
def test_stored_results_match_the_tree(name):
    g = load_golden(name)                     # asserts the digest
    assert len(golden_source_digest()) == 64
    wl = WL.WORKLOADS[name]
    idx = g["index"]
    assert idx[0] == 0 and idx[-1] == wl.n_params - 1 and np.all(np.diff(idx) > 0)
    for tag in ("bf16", "exact"):
        assert g[tag + "_params"].shape == idx.shape and np.isfinite(g[tag + "_params"]).all()
        assert g[tag + "_max_abs_update"] > 0
    if name == "batch4":
        assert g["bf16_losses"].shape == (wl.steps + 1,) and g["exact_mious"].shape == (wl.steps + 1, wl.n)
        # the two oracle modes differ by the bfloat16 rounding of the operands and no more
        assert np.abs(g["bf16_losses"] - g["exact_losses"]).max() < 2e-3
        assert np.all(np.diff(g["exact_losses"]) < 0)          # sixteen descent steps at lr 0.005
    else:
        assert g["bf16_scores"].shape == (32,) and g["bf16_key"].all() and (g["exact_updates"] == wl.steps).all()
