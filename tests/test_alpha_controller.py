"""The split controller (paper Sec. IV-A) on the CPU: its steps come from the action set of Eq. 3, the
fraction obeys the update rule and the bounds of Eq. 4 / Eq. 6, the reward is Eq. 5, the Recovery Controller
fires as the paper states it, and the stand-in policy (a hill climb on latency; the paper's trained policy
is not available, so nothing here is parity with it) finds the minimum of a U-shaped latency curve.  The
decisions are applied to a metadata-only pool through pool_set_split."""
import numpy as np
import pytest

from paper_2605_04450_amd import binding as B
from tests.test_oracle_pool import golden

ACTIONS = (-0.06, -0.04, -0.02, 0.0, 0.02, 0.04, 0.06)


def latency(alpha, best, rng=None, noise=0.0):
    """A U-shaped latency in ms with its minimum at `best` (the shape of the paper's Sec. III trade-off)."""
    v = 12.0 + 160.0 * (alpha - best) ** 2
    return v * (1.0 + (rng.normal(0.0, noise) if rng is not None else 0.0))


def test_action_set_and_bounds_are_the_papers():
    g = golden()  # tests/golden/paper_closed_forms.txt: values printed in the paper
    assert (g["alpha_min"], g["alpha_max"], g["alpha_step"], g["action_max"], g["action_count"]) == (0.1, 0.9, 0.02, 0.06, 7)
    assert sorted(ACTIONS) == [round(g["alpha_step"] * k, 2) for k in range(-3, 4)] and len(ACTIONS) == g["action_count"]
    rng = np.random.default_rng(0)
    ctl = B.AlphaController(30.0)
    alpha = 0.5
    for t in range(300):  # arbitrary observations: whatever the policy sees, its answer is a legal action
        lat = float(rng.uniform(5.0, 80.0))
        step, nxt, burst = ctl.decide(alpha, lat, hot_user_ratio=float(rng.uniform()), kv_hit_rate=float(rng.uniform()),
                                      emb_hit_rate=float(rng.uniform()))
        assert min(abs(step - a) for a in ACTIONS) < 1e-12, step
        assert g["alpha_min"] <= nxt <= g["alpha_max"]
        assert nxt == pytest.approx(min(g["alpha_max"], max(g["alpha_min"], alpha + step)), abs=1e-12)  # Eq. 4
        alpha = nxt


@pytest.mark.parametrize("start,best", [(0.8, 0.34), (0.2, 0.55), (0.5, 0.1), (0.12, 0.9)])
def test_hill_climb_settles_at_the_minimum_of_a_u_shaped_latency(start, best):
    ctl = B.AlphaController(30.0)
    rng = np.random.default_rng(4)
    rc, pool = B.pool_create(None, 4096 * 64, 64, 16, B.ELEM_F32, 4, 32, None, 0, start)  # metadata only
    assert rc == B.OK
    alpha, path = start, []
    for t in range(80):
        step, nxt, burst = ctl.decide(alpha, latency(alpha, best, rng, 0.002), kv_hit_rate=0.5, emb_hit_rate=0.4 if best > start else 0.6)
        assert not burst
        if nxt != alpha:
            rc, ach = B.pool_set_split(pool, nxt, device=False)
            assert rc == B.OK and B.pool_stats(pool)["pages_emb"] == round(nxt * 4096)
            assert ach == pytest.approx(nxt, abs=1.0 / 4096)
        alpha = nxt
        path.append(alpha)
    # it stops where one more step changes the latency by less than its 2 % tolerance: within 0.08 of the minimum
    assert max(abs(a - best) for a in path[-20:]) <= 0.08 + 1e-9, path[-20:]
    assert latency(path[-1], best) <= 1.08 * latency(best, best)
    B.pool_destroy(pool)


def test_recovery_controller_overrides_on_a_burst():
    for hot, want in ((0.35, -0.06), (0.1, 0.0)):
        ctl = B.AlphaController(30.0)
        alpha = 0.5
        rng = np.random.default_rng(1)
        for t in range(12):
            step, alpha, burst = ctl.decide(alpha, 20.0 + float(rng.normal(0.0, 0.1)), hot_user_ratio=hot)
            assert not burst
        step, alpha, burst = ctl.decide(alpha, 22.5, hot_user_ratio=hot)  # within three times the floor (5 % of 20 ms)
        assert not burst
        step, nxt, burst = ctl.decide(alpha, 26.0, hot_user_ratio=hot)    # beyond it
        assert burst and step == want and nxt == pytest.approx(max(0.1, alpha + want))
    ctl = B.AlphaController(30.0)
    for t in range(12):  # a steady ramp is not a burst: every epoch stays within three sigma of the window's mean
        step, alpha, burst = ctl.decide(0.5, 20.0 + 0.5 * t)
        assert not burst


def test_reward_is_slo_satisfaction_less_the_tail_penalty():
    assert B.alpha_reward(0.9, 36.0, 30.0) == pytest.approx(0.9 - 6.0 / 30.0)   # Eq. 5 with lambda = 1 / tau
    assert B.alpha_reward(0.97, 25.0, 30.0) == pytest.approx(0.97)             # no penalty below the SLO
    assert B.alpha_reward(1.0, 30.0, 30.0) == 1.0


def test_argument_errors():
    with pytest.raises(ValueError):
        B.AlphaController(0.0)
    ctl = B.AlphaController(30.0)
    with pytest.raises(ValueError):
        ctl.decide(1.5, 10.0)
    with pytest.raises(ValueError):
        ctl.decide(0.5, -1.0)
