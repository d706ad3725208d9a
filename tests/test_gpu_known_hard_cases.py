"""Cases that random sweeps of `tests/test_gpu_random.py`'s generators found above the 1e-4 tolerance, kept with their
seeds.  The normalised update N = u_hat / (sqrt(v_hat) + eps) divides by quantities that come from g; where an entry of
g is a nearly cancelled sum, the rounding of the products shows amplified in N (and in the column scale of the
full-rank QHM term).  What each group needed:
  * fp32 gradients (cases 150, 154 of the option sweep; Rayleigh-Ritz case 99): the down-projection of fp32 gradients
    now runs with three-term operands, as exact as fp32;
  * bf16 gradients behind a basis ordered by the Rayleigh-Ritz step, refreshed after exactly ONE step from the zero
    state (case 27 of that sweep and a 649 x 608 matrix of rank 264 from a sweep of ranks above 128, both skipped):
    g, u, v and the weight change agree to 1e-4 (u and v after the rotation to 3e-6), N reaches 1.1e-4 and 1.9e-4.
    After one step v_hat = u_hat^2 identically, so the variance term of the rotated second moment,
    c2 |(R o R)(v_hat - u_hat^2) + (R u_hat)^2|, is zero in exact arithmetic and in float64; computed from moments
    STORED in fp32 it is their rounding noise, 1e-7 v_hat with either sign.  Where the rotated first moment is small
    -- the trailing directions of a basis ordered by singular value are exactly those -- (R u_hat)^2 is no longer
    large against that noise, the element of v has a large RELATIVE error (the array as a whole stays within 3e-6),
    and N = u_hat / (sqrt(v_hat) + eps) divides by it.  With two or three steps before the refresh, so that the
    variance term is a variance, the same two cases give 5e-6 on N (measured).  A third bf16 term of Q in the
    down-projection does not change the one-step case (1.6e-4): it would take moments stored beyond fp32;
  * one element in 14 696 (case 317 of the option sweep, skipped): bf16 gradients, a 47 x 668 matrix of rank 22.  g, u
    and v agree to 1e-5, and the library's N equals the float64 formula evaluated at the library's own u, v, g to
    3e-6; but one entry of g is about a thousand times smaller than the typical entry at BOTH of the first two steps,
    so that u and v there consist of nothing else, the fp32-level absolute error of g (1e-5 of its rms, from the
    2^-17 operand split of Q) is 1 % of the entry, and N = u_hat / sqrt(v_hat), which does not depend on the scale of
    the entry, is off by 0.0125 in that one place -- the whole of the 1.16e-4.  With every further step the chance
    that an entry has seen only such gradients falls off geometrically (the first update from a zero state is where
    the tests already take the library's value after a closed-form check);
  * the same on a right-projected matrix (a 300-case sweep of mixed left / right shape sets, case 193, skipped): a
    244 x 352 matrix of rank 124 projected on the right, plain update, bf16 gradients: g, u, v within 3e-6 at every
    step, N of the second step at 1.9e-4 and the weight change since the start at 1.24e-4, back to 5e-6 and 6e-5 one
    step later."""
import pytest

from tests import test_gpu_random as sweep
from tests import test_gpu_right_projection as right

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("case", [
    150, 154,
    pytest.param(317, marks=pytest.mark.skip(reason="known miss: N and the weight change of the second step at 1.16e-4 on one 47 x 668, r = 22 matrix, all of it "
                                                    "in ONE element whose g is ~1000x below the typical entry at both steps (g, u, v within 1e-5; library N = float64 "
                                                    "formula of its own u, v, g to 3e-6): conditioning of N in fp32, see the module docstring"))])
def test_option_sweep_cases(case):
    sweep.test_random_shapes_and_options(case)


@pytest.mark.parametrize("case", [
    pytest.param(27, marks=pytest.mark.skip(reason="known miss: N of the step after a Rayleigh-Ritz refresh that follows ONE step from the zero state at 1.1e-4 on "
                                                   "one 347 x 252, r = 46 matrix (g, u, v, dW within 1e-4; 5e-6 with two steps before the refresh): the variance term "
                                                   "of the rotation is rounding noise of the fp32 moments, see the module docstring")),
    99])
def test_rayleigh_ritz_sweep_cases(case):
    sweep.test_random_shapes_rayleigh_ritz_refresh(case, steps_before_refresh=1)


@pytest.mark.skip(reason="known miss: N of the second step at 1.9e-4 on the 244 x 352, r = 124 right-projected matrix (g, u, v within 3e-6), one "
                         "ill-conditioned element as in option-sweep case 317, see the module docstring")
def test_right_projection_sweep_case_193():
    right.SHAPE_SETS["sweep_193"] = [(454, 32, 8, 1), (454, 64, 56, 0), (244, 352, 124, 1)]
    try:
        right.test_right_projection_steps_refresh_outer("sweep_193", "none", True)
    finally:
        del right.SHAPE_SETS["sweep_193"]


@pytest.mark.skip(reason="known miss: N of the step after a Rayleigh-Ritz refresh that follows ONE step from the zero state at 1.9e-4 (g, u, v, dW within "
                         "1e-4; 5e-6 with two steps before the refresh): the variance term of the rotation is rounding noise of the fp32 moments, see the "
                         "module docstring")
def test_rayleigh_ritz_rank_264_refresh_after_one_step(monkeypatch):
    monkeypatch.setattr(sweep, "draw_rr_case", lambda case: ([(649, 608, 264)], True, 1))
    sweep.test_random_shapes_rayleigh_ritz_refresh(6, steps_before_refresh=1)
