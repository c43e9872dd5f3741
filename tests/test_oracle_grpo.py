"""Pins of the reference GRPO advantage (mean / standard-deviation normalisation within the
samples of one prompt; Shao et al. 2024, used by the paper, Section 8.1): closed forms and
invariants, none of which retypes the reference's formula."""
import numpy as np

from oracle import reference as R


def test_two_member_group_is_plus_minus_one():
    # deviations of {a, b} are +-(a-b)/2 and the standard deviation is |a-b|/2
    adv = R.grpo_advantages([3.0, 7.0, -1.0, -1.5], [0, 0, 1, 1], 2, 0.0)
    np.testing.assert_allclose(adv, [-1.0, 1.0, 1.0, -1.0], atol=1e-15)


def test_equal_rewards_give_zero_and_singletons_too():
    adv = R.grpo_advantages([2.0, 2.0, 2.0, 5.0], [0, 0, 0, 1], 2, 0.0)
    np.testing.assert_array_equal(adv, np.zeros(4))
    adv = R.grpo_advantages([2.0, 2.0, 2.0, 5.0], [0, 0, 0, 1], 2, 1e-4)
    np.testing.assert_array_equal(adv, np.zeros(4))


def test_worked_example_one_success_in_four():
    # rewards (1,0,0,0): mean 1/4, variance 3/16 -> advantages sqrt(3) and -1/sqrt(3)
    adv = R.grpo_advantages([1.0, 0.0, 0.0, 0.0], [0, 0, 0, 0], 1, 0.0)
    np.testing.assert_allclose(adv, [np.sqrt(3.0)] + [-1.0 / np.sqrt(3.0)] * 3, rtol=1e-15)


def test_normalised_moments_and_affine_invariance():
    rng = np.random.default_rng(11)
    NG, G = 7, 9
    gos = rng.permutation(np.repeat(np.arange(NG), G))
    r = rng.normal(size=NG * G)
    adv = R.grpo_advantages(r, gos, NG, 0.0)
    for g in range(NG):
        a = adv[gos == g]
        assert abs(a.mean()) < 1e-14
        assert abs((a * a).mean() - 1.0) < 1e-13
    # positive affine maps of the rewards leave the advantages alone, a negative scale flips them
    np.testing.assert_allclose(R.grpo_advantages(4.0 * r + 3.0, gos, NG, 0.0), adv, atol=1e-12)
    np.testing.assert_allclose(R.grpo_advantages(-0.5 * r, gos, NG, 0.0), -adv, atol=1e-12)
    # groups are independent: changing one group's rewards changes only that group
    r2 = r.copy()
    r2[gos == 3] += rng.normal(size=G)
    adv2 = R.grpo_advantages(r2, gos, NG, 0.0)
    np.testing.assert_array_equal(adv2[gos != 3], adv[gos != 3])


def test_eps_shrinks_towards_zero_by_the_stated_factor():
    r = np.array([0.0, 2.0, 4.0, 6.0])          # deviations -3,-1,1,3; std = sqrt(5)
    adv = R.grpo_advantages(r, [0, 0, 0, 0], 1, 0.5)
    np.testing.assert_allclose(adv, np.array([-3.0, -1.0, 1.0, 3.0]) / (np.sqrt(5.0) + 0.5), rtol=1e-15)


def test_sequences_without_group_are_nan():
    adv = R.grpo_advantages([1.0, 2.0, 3.0], [0, -1, 0], 1, 0.0)
    assert np.isnan(adv[1]) and adv[0] == -1.0 and adv[2] == 1.0
