"""Host-side logic of libfae that needs no GPU: the Student-t quantile used by the
confidence interval (Sec. 4.1.2, Eq. 4) and the Shuffle Scheduler rate rule (Sec. 5,
Eq. 5), each against the oracle."""
import numpy as np
import pytest

from oracle import fae_oracle as O
from paper_2103_00686_amd import binding as B


@pytest.mark.parametrize("confidence", [0.5, 0.9, 0.95, 0.99, 0.999, 0.99999])
@pytest.mark.parametrize("n", [2, 3, 5, 11, 35, 36, 200, 10_001])
def test_t_quantile_matches_the_oracle(confidence, n):
    got = B.fae_t_quantile(confidence, n - 1)
    ref = O.t_quantile(confidence, n)
    assert abs(got - ref) <= 1e-8 * ref


def test_t_quantile_rejects_bad_arguments():
    assert B.fae_t_quantile(1.0, 5) < 0 and B.fae_t_quantile(0.0, 5) < 0 and B.fae_t_quantile(0.9, 0) < 0


@pytest.mark.parametrize("seed", range(8))
def test_scheduler_follows_the_oracle_on_random_loss_curves(seed):
    rng = np.random.default_rng(seed)
    # a noisy falling curve with plateaus (exact repeats) and bumps
    losses = np.round(2.0 * np.exp(-np.arange(60) / 25.0) + 0.05 * rng.standard_normal(60), 2).tolist()
    for u, p0 in ((4, 50.0), (2, 50.0), (4, 3.0), (1, 100.0)):
        s = B.Sched(p0, u)
        got = [s.report(x) for x in losses]
        assert got == O.shuffle_scheduler(losses, p0, u)
        assert all(1.0 <= r <= 100.0 for r in got)


def test_scheduler_segments_and_arguments():
    s = B.Sched()                          # the paper's start: R(50), u = 4
    assert s.rate == 50.0
    assert s.segment(1000) == 500 and s.segment(3) == 2 and s.segment(1) == 1 and s.segment(0) == 0
    for _ in range(10):
        s.report(1.0)                      # never falling: down to R(1)
    assert s.rate == 1.0 and s.segment(1000) == 10 and s.segment(50) == 1
    with pytest.raises(B.FaeError):
        B.Sched(0.5, 4)
    with pytest.raises(B.FaeError):
        B.Sched(50.0, 0)
    with pytest.raises(B.FaeError):
        s.report(float("nan"))
