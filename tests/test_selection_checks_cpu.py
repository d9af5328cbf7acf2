"""The checkers that judge a GPU selection which differs from the oracle's are themselves checked
here, on the CPU: a correct row passes, and each kind of wrong row (planted on the CPU) is caught."""
import numpy as np
import pytest
import torch

from oracle import superlinear as orc
from oracle.checks import selection_problems
from tests import brute

MARGIN = 1e-3


def test_selection_problems_accepts_the_oracle_row_and_margin_swaps():
    s = np.array([0.5, 3.0, 2.0, 2.0004, -1.0, 2.9])
    want = orc.select_topk(s, 3)                       # spans 1, 3, 5
    assert want == [1, 3, 5]
    assert selection_problems(s, want, 3, MARGIN) == []
    # span 2 scores 0.0004 below span 3: inside the margin, either may be listed
    assert selection_problems(s, [1, 2, 5], 3, MARGIN) == []
    # fewer candidates than slots: everything listed, -1 padding
    assert selection_problems(s[:2], [0, 1, -1], 3, MARGIN) == []
    assert selection_problems(s[:0], [-1, -1], 2, MARGIN) == []


@pytest.mark.parametrize("row,why", [
    ([0, 1, 5], "below"),          # span 0 scores 1.5 below the k-th score
    ([1, 4, 5], "below"),
    ([1, 5, 3], "ascending"),      # right set, wrong order
    ([1, 1, 5], "twice"),
    ([1, 5, -1], "expected min"),  # one missing
    ([-1, 1, 5], "empty slots"),   # padding in front
    ([1, 5, 6], "out of range"),
    ([1, 3], "slots"),
])
def test_selection_problems_rejects_wrong_rows(row, why):
    s = np.array([0.5, 3.0, 2.0, 2.0004, -1.0, 2.9])
    problems = selection_problems(s, row, 3, MARGIN)
    assert problems and any(why in p for p in problems), problems


def test_selection_problems_dropped_span_above_margin():
    # a row that picks only spans near the k-th score but drops the clear winner
    s = np.array([5.0, 2.0, 2.0003, 2.0006])
    problems = selection_problems(s, [1, 2], 2, MARGIN)
    assert any("dropped" in p for p in problems)


def _case(seed=3, Hq=4, Hkv=2, L=900, D=32, S=32, k=5, q_pos0=0, Lq=None):
    g = torch.Generator().manual_seed(seed)
    Lq = L if Lq is None else Lq
    Qs = torch.randn((Hq, Lq, D), generator=g, dtype=torch.float64)
    K = torch.randn((Hkv, L, D), generator=g, dtype=torch.float64)
    Ks = torch.from_numpy(orc.span_keys(K.numpy(), S))
    idx = torch.from_numpy(orc.span_search(Qs.numpy(), Ks.numpy(), S, k, q_pos0=q_pos0).astype(np.int32))
    return idx, Qs, Ks


@pytest.mark.parametrize("q_pos0,Lq", [(0, None), (500, 400)])
def test_all_rows_check_accepts_the_oracle(q_pos0, Lq):
    idx, Qs, Ks = _case(q_pos0=q_pos0, Lq=Lq)
    rows, differ = brute.check_selection_all_rows(idx, Qs, Ks, 32, 5, q_pos0=q_pos0, margin=MARGIN, chunk=256)
    assert rows == idx.shape[0] * idx.shape[1] and differ == 0


def test_all_rows_check_accepts_exact_ties_resolved_to_the_lower_index_only():
    idx, Qs, Ks = _case()
    Ks[:, 7] = Ks[:, 3]            # spans 3 and 7 tie exactly for every query
    idx = torch.from_numpy(orc.span_search(Qs.numpy(), Ks.numpy(), 32, 5).astype(np.int32))
    _, differ = brute.check_selection_all_rows(idx, Qs, Ks, 32, 5, margin=MARGIN)
    assert differ == 0
    # swapping 3 for 7 where only 3 was selected stays inside the margin: accepted, but counted
    swapped = idx.clone()
    n_swapped = 0
    for h in range(idx.shape[0]):
        for r in range(idx.shape[1]):
            row = idx[h, r].tolist()
            if 3 in row and 7 not in row and r // 32 > 7:
                new = sorted([7 if j == 3 else j for j in row if j >= 0])
                swapped[h, r] = torch.tensor(new + [-1] * (5 - len(new)), dtype=torch.int32)
                n_swapped += 1
    assert n_swapped > 0
    _, differ = brute.check_selection_all_rows(swapped, Qs, Ks, 32, 5, margin=MARGIN)
    assert differ == n_swapped


@pytest.mark.parametrize("mistake", ["wrong_span", "unsorted", "duplicate", "missing", "own_span", "pad_first"])
def test_all_rows_check_catches_planted_mistakes(mistake):
    idx, Qs, Ks = _case()
    h, r = 2, 700                                       # c = 21 candidates, 5 selected
    row = idx[h, r].tolist()
    if mistake == "wrong_span":
        worst = int(torch.argmin(Qs[h, r] @ Ks[h // 2, :21].T))
        row = sorted([worst] + row[1:]) if worst not in row else row[::-1]
    elif mistake == "unsorted":
        row = row[::-1]
    elif mistake == "duplicate":
        row[1] = row[0]
    elif mistake == "missing":
        row[-1] = -1
    elif mistake == "own_span":
        row[-1] = 21
    elif mistake == "pad_first":
        row = [-1] + row[:-1]
    idx[h, r] = torch.tensor(row, dtype=torch.int32)
    with pytest.raises(AssertionError):
        brute.check_selection_all_rows(idx, Qs, Ks, 32, 5, margin=MARGIN)
