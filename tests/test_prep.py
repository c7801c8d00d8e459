"""Input preparation (allocation thresholds of Section 3.2 / Appendix A, reorder)."""
import math
import os

import numpy as np
import pytest
import torch

from paper_2602_08923_amd import prep, workloads


def gold(golden_dir):
    vals = {}
    with open(os.path.join(golden_dir, "paper_worked_examples.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, val, _ = [s.strip() for s in line.split("|", 2)]
            vals[name] = float(val)
    return vals


def per_bit_benefit(T, a, b):
    # Section 3.2: T * (4^(b-a) - 1) / (4^b * (b - a))
    return T * (4 ** (b - a) - 1) / (4 ** b * (b - a))


def test_threshold_ratios_follow_from_equal_per_bit_benefit(golden_dir):
    g = gold(golden_dir)
    assert per_bit_benefit(1.0, 1, 2) == 3 / 16
    assert per_bit_benefit(1.0, 2, 4) == 15 / 512
    assert per_bit_benefit(1.0, 4, 8) == 255 / 4 ** 9
    assert per_bit_benefit(1.0, 2, 4) / per_bit_benefit(1.0, 1, 2) == g["threshold_ratio_1_2"] == 5 / 32
    assert per_bit_benefit(1.0, 4, 8) / per_bit_benefit(1.0, 2, 4) == g["threshold_ratio_2_4"] == 17 / 512
    assert per_bit_benefit(1.0, 8, 16) / per_bit_benefit(1.0, 4, 8) == g["threshold_ratio_4_8"] == 257 / 2 ** 17


def test_allocation_rule_thresholds():
    # z(T48) - z(T24) = 4 when T24 = 17/512 T48 (Appendix A)
    assert prep.K_ALLOC * math.log2(512 / 17) == pytest.approx(4.0)
    F = torch.tensor([2.0 ** -30, 2.0 ** -20, 2.0 ** -10, 0.0], dtype=torch.float64)
    u = 4.0 - prep.K_ALLOC * math.log2(2.0 ** -20)  # puts the 2|4 threshold exactly at F = 2^-20
    q = prep.widths_for_offset(F, u)
    assert q.tolist() == [2.0, 4.0, 8.0, 2.0]


@pytest.mark.parametrize("budget", [3.0, 4.0, 5.0])
def test_allocation_meets_budget_tightly(budget):
    g = torch.Generator().manual_seed(1)
    F = torch.exp(torch.randn(4096, generator=g, dtype=torch.float64) * 3.0)
    w = prep.allocate(F, budget)
    avg = float(w.double().mean())
    assert avg <= prep.code_bits(budget) and avg > prep.code_bits(budget) - 0.01
    # monotone: a larger F never gets fewer bits
    order = torch.argsort(F)
    assert torch.all(w[order][1:] >= w[order][:-1])


def test_code_bits_matches_paper(golden_dir):
    assert prep.code_bits(5.0) == gold(golden_dir)["budget5_code_bits"]


def test_reorder_roundtrip_and_counts():
    w = torch.tensor([4, 2, 8, 4, 2, 4, 4, 8])
    perm, counts = prep.reorder_plan(w, 4)
    assert counts == [2, 4, 2] and perm.tolist() == [1, 4, 0, 3, 5, 6, 2, 7]
    x = torch.arange(8 * 256, dtype=torch.float32)
    y = prep.apply_reorder(x, perm)
    assert y[:256].tolist() == x[256:512].tolist()
    assert torch.equal(prep.undo_reorder(y, perm), x)
    assert prep.chunk_counts(counts, 4) == [[2, 0, 0], [0, 2, 0], [0, 2, 0], [0, 0, 2]]


def test_workloads_are_seeded_and_shaped():
    for cid in (1, 2, 4, 5):
        wl = workloads.CONFIGS[cid]
        a = workloads.draw(wl, 1, 0, entries=4096)
        b = workloads.draw(wl, 1, 0, entries=4096)
        c = workloads.draw(wl, 2, 0, entries=4096)
        assert torch.equal(a, b) and not torch.equal(a, c)
        assert a.dtype == (torch.float32 if wl.dtype == "f32" else torch.bfloat16)
    x = workloads.draw(workloads.CONFIGS[2], 0, 0, entries=1 << 18).float()
    assert 0.5e-3 < float(x.abs().median()) / 0.6745 < 1.5e-3
    assert float(x.abs().max()) > 0.05  # the x100 outliers are there
    h = workloads.to_numpy(workloads.draw(workloads.CONFIGS[2], 0, 0, entries=512))
    assert h.dtype == np.uint16
