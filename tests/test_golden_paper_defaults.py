"""The hyper-parameters the paper prints (tests/golden/paper_defaults.json, with its citation) against the
defaults of the oracle and of the binding, and what they imply for Algorithm 2's termination."""
import inspect
import json
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_defaults.json")


@pytest.fixture(scope="module")
def paper():
    return json.load(open(GOLDEN))


def test_default_update_ratios_are_the_papers(orc, paper):
    from paper_2602_17698_amd import binding as sb
    sig = inspect.signature(orc.allocate).parameters
    assert sig["gamma0"].default == paper["gamma0"] and sig["gammaT"].default == paper["gammaT"]
    sig = inspect.signature(sb.Plan.allocate).parameters
    assert sig["gamma0"].default == paper["gamma0"] and sig["gammaT"].default == paper["gammaT"]
    header = open(os.path.join(os.path.dirname(GOLDEN), "..", "..", "include", "scalebits.h")).read()
    assert "paper: 0.05" in header and "paper: 0.02" in header


@pytest.mark.parametrize("N", [400, 1000, 4096, 26624])
def test_search_in_the_papers_space_ends_at_the_second_rejected_swap(orc, paper, N):
    bits = paper["bitwidths"]
    rng = np.random.default_rng(N)
    sens = np.exp(2.0 * rng.normal(size=(N, 1)))
    cost = (sens * 4.0 ** -np.asarray(bits, np.float64)[None, :] * np.exp(0.2 * rng.normal(size=(N, len(bits))))).astype(np.float32)
    rc, level, st, tr = orc.allocate(cost, bits, 3.0, want_trace=True)          # default ratios = the paper's
    assert rc == 0
    k0 = int(np.floor(paper["gamma0"] * N))
    assert tr[0]["k"] == k0
    assert st["swaps_rej"] == paper["rejections_until_stop"]
    assert tr[-1]["kind"] == 2                                                   # the last iteration is a rejected swap
    assert st["k_final"] == k0 // 2 // 2 < int(np.floor(paper["gammaT"] * N)) <= k0 // 2
    assert st["bits_used"] <= st["bits_budget"] == 3 * N


def test_both_mixtures_of_the_kernel_table_are_four_bits(orc):
    """The two rows of the paper's kernel-latency table store the same number of bytes: the stream's
    offsets for each mixture end at rows * cols * 4 / 8 (tiles of 128 x 128, counts rounded as bench.py does)."""
    t = json.load(open(os.path.join(os.path.dirname(GOLDEN), "kernel_table_mixtures.json")))
    m = n = 128
    N = (t["rows"] // m) * (t["cols"] // n)
    for mix in t["mixtures"]:
        counts = [int(round(f * N)) for f in mix]
        counts[1] += N - sum(counts)
        level = np.random.default_rng(0).permutation(np.repeat(np.arange(3, dtype=np.uint8), counts))
        off = orc.offsets(level, m, n, t["bitwidths"])
        assert int(off[-1]) == t["rows"] * t["cols"] * t["average_bits"] // 8
        assert np.all(np.diff(off) == (np.asarray(t["bitwidths"])[level] * (m * n // 8)))
