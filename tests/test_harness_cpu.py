"""The comparison rules of the GPU parity tests, exercised on the CPU with planted mistakes:
every rule must accept what it should and reject a wrong result."""
import numpy as np
import pytest
import torch

import oracle
from tests import harness as Hn
from tests.test_oracle_pins import make_case


def test_selection_rule_accepts_exact_and_band_swaps_only():
    s = np.array([5.0, 1.0, 4.0, 3.0, 3.0 + 1e-6, 0.5, 2.0])
    k = 3
    exact = np.array([0, 2, 4, -1], np.int32)          # 5, 4, 3+1e-6
    assert Hn.check_selection_row(exact[:k + 1][:4], 3, s, 3) in (True,)
    # page 3 (score 3.0) is within 1e-4 relative of the k-th score: swapping it in is a legitimate near-tie
    swapped = np.array([0, 2, 3], np.int32)
    assert Hn.check_selection_row(swapped, 3, s, 3) is False
    with pytest.raises(AssertionError):                 # page 6 (score 2.0) is far below the band
        Hn.check_selection_row(np.array([0, 2, 6], np.int32), 3, s, 3)
    with pytest.raises(AssertionError):                 # a clearly better page is missing
        Hn.check_selection_row(np.array([2, 3, 4], np.int32), 3, s, 3)
    with pytest.raises(AssertionError):                 # duplicates / not ascending
        Hn.check_selection_row(np.array([0, 2, 2], np.int32), 3, s, 3)
    with pytest.raises(AssertionError):                 # wrong count
        Hn.check_selection_row(np.array([0, 2, 4], np.int32), 2, s, 3)
    with pytest.raises(AssertionError):                 # out of range
        Hn.check_selection_row(np.array([0, 2, 9], np.int32), 3, s, 3)
    with pytest.raises(AssertionError):                 # padding must be -1
        Hn.check_selection_row(np.array([0, 2, 4, 0], np.int32), 3, s, 3)
    # a clear gap forces the oracle's set exactly
    s2 = np.array([5.0, 1.0, 4.0, 3.0, 2.0])
    with pytest.raises(AssertionError):
        Hn.check_selection_row(np.array([0, 2, 4], np.int32), 3, s2, 3)
    # k >= P: all pages
    assert Hn.check_selection_row(np.array([0, 1, 2, 3, 4, -1], np.int32), 5, s2, 6)


def test_selection_rule_with_always_kept_pages():
    s = np.array([5.0, 1.0, 4.0, 3.0, 0.2, 0.1, 0.3])          # the last two pages score lowest
    # k = 4, the last 2 pages forced: {5, 6} plus the best two of the rest {0, 2}
    assert Hn.check_selection_row(np.array([0, 2, 5, 6], np.int32), 4, s, 4, force_recent=2)
    assert Hn.check_selection_row(np.array([0, 2, 5, 6, -1], np.int32), 4, s, 4, force_recent=2)
    with pytest.raises(AssertionError):                 # plain top-4 ignores the forced pages
        Hn.check_selection_row(np.array([0, 2, 3, 6], np.int32), 4, s, 4, force_recent=2)
    with pytest.raises(AssertionError):                 # forced pages there, but the rest is not the best of the others
        Hn.check_selection_row(np.array([0, 3, 5, 6], np.int32), 4, s, 4, force_recent=2)
    with pytest.raises(AssertionError):                 # the same set is wrong when nothing is forced
        Hn.check_selection_row(np.array([0, 2, 5, 6], np.int32), 4, s, 4)
    # n >= k: exactly the last k pages
    assert Hn.check_selection_row(np.array([4, 5, 6], np.int32), 3, s, 3, force_recent=5)
    with pytest.raises(AssertionError):
        Hn.check_selection_row(np.array([0, 5, 6], np.int32), 3, s, 3, force_recent=5)


def test_attention_rule_flags_a_wrong_output():
    c, q = make_case(21, lens=(13, 7))
    pages = [0, 2]
    o, lse = oracle.attention(c, q, 0, 1, pages)
    out = torch.zeros((c.B, c.H, c.D))
    lse_t = torch.zeros((c.B, c.H))
    out[0, 1] = torch.from_numpy(o).float()
    lse_t[0, 1] = lse
    Hn.check_attention_head(out, lse_t, c, q, 0, 1, pages, torch.float32)
    bad = out.clone()
    bad[0, 1, 3] += 5e-4
    with pytest.raises(AssertionError):
        Hn.check_attention_head(bad, lse_t, c, q, 0, 1, pages, torch.float32)
    with pytest.raises(AssertionError):                 # attended the wrong page set
        Hn.check_attention_head(out, lse_t, c, q, 0, 1, [0, 3], torch.float32)
    bad_lse = lse_t.clone()
    bad_lse[0, 1] += 1e-2
    with pytest.raises(AssertionError):
        Hn.check_attention_head(out, bad_lse, c, q, 0, 1, pages, torch.float32)


def test_bf16_mean_rule_accepts_the_oracle_rounding_and_justified_neighbours_only():
    """Stored bf16 means have to be the oracle's float64 means rounded once; a neighbouring bf16 value passes only
    where the float64 mean sits within the fp32 accumulation bound of the rounding boundary."""
    rng = np.random.default_rng(5)
    mean = rng.normal(size=(6, 16)) * 0.5
    n_keys, abs_mean = 16.0, 0.8
    akm = lambda idx: (np.full(idx[0].shape, abs_mean), np.full(idx[0].shape, n_keys))
    good = oracle.round_bf16(mean)
    used, (n, worst) = Hn.check_bf16_means(good.copy(), mean, akm)
    assert n == 0 and worst == 0.0 and np.array_equal(used, oracle.bf16_to_double(good))
    # a neighbour where the mean is far from the boundary: rejected
    bad = good.copy()
    bad[2, 3] += 1
    with pytest.raises(AssertionError):
        Hn.check_bf16_means(bad, mean, akm)
    # two values away: rejected whatever the mean
    bad2 = good.copy()
    bad2[1, 1] += 2
    with pytest.raises(AssertionError):
        Hn.check_bf16_means(bad2, mean, akm)
    # a mean placed 1e-7 of its size beside a rounding boundary: both neighbours pass, and the one the kernel stored is
    # what the later stages are checked with
    lo, hi = oracle.bf16_to_double(np.array([0x3F00, 0x3F01], np.uint16))      # 0.5 and the next bf16 value
    mean2 = mean.copy()
    mean2[4, 7] = 0.5 * (lo + hi) + 2e-8
    want = oracle.round_bf16(mean2)
    assert want[4, 7] == 0x3F01
    other = want.copy()
    other[4, 7] = 0x3F00
    used, (n, worst) = Hn.check_bf16_means(other, mean2, akm)
    assert n == 1 and 0 < worst <= 1.0 and used[4, 7] == lo
    # the same neighbour with the mean 1e-5 away from the boundary: outside the bound, rejected
    mean2[4, 7] = 0.5 * (lo + hi) + 1e-5
    with pytest.raises(AssertionError):
        Hn.check_bf16_means(other, mean2, akm)
    # keys that cancel: a float64 mean of 2e-9 under a bound of 8.6e-7. An fp32 sum of the same keys may land anywhere
    # within the bound, also on the other side of zero, many bf16 values away from the oracle's rounding: accepted;
    # a stored value beyond the bound is not
    mean3 = mean.copy()
    mean3[0, 0] = 2e-9
    want3 = oracle.round_bf16(mean3)
    for v, fine in ((-3e-7, True), (5e-7, True), (0.0, True), (-2e-6, False), (3e-6, False)):
        stored = want3.copy()
        stored[0, 0] = oracle.round_bf16(np.array([v]))[0]
        if fine:
            used, (n, worst) = Hn.check_bf16_means(stored, mean3, akm)
            assert n == 1 and 0 < worst <= 1.0 and used[0, 0] == oracle.bf16_to_double(stored[0:1, 0])[0]
        else:
            with pytest.raises(AssertionError):
                Hn.check_bf16_means(stored, mean3, akm)
