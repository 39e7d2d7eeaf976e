"""Host-side MDP agent (Section 3.3, Algorithm 2): the library's C++ against a hand-computed example,
the paper's stated properties, and the plain numpy restatement in oracle/mdp_ref.py.  CPU only.

What stays unpinned: the learning dynamics depend on values the paper does not give (SARSA discount,
weight initialisation, input normalisation); they are checked only for agreement between the two
independent implementations of the same readings."""
import os

import numpy as np
import pytest

from oracle import mdp_ref
from paper_1804_08066_amd import mqgrad, workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "mdp_worked_example.txt")


def golden():
    d = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        d[k] = [float(t) for t in v]
    return d


def test_reference_statistics_match_the_hand_computed_example():
    g = golden()
    sm = mdp_ref.moving_average(g["losses"], g["alpha"][0], g["start"][0])
    assert sm == g["smoothed"]
    assert abs(mdp_ref.slope(g["smoothed"]) - g["beta"][0]) < 1e-12
    assert abs(-(1 / g["cost_ms"][0]) * mdp_ref.slope(g["smoothed"]) * g["gamma"][0] - g["reward"][0]) < 1e-12


def test_library_moving_average_slope_and_reward_match_the_hand_computed_example():
    g = golden()
    # first loss 4 makes the running average start at 4 (the example's previous smoothed value)
    agent = mqgrad.Mdp(alpha=g["alpha"][0], window=5, decide_every=5, reward_scale=g["gamma"][0], epsilon=0.0)
    agent.step(4.0, 0.0)                       # iteration 0: first decision, no reward yet
    assert agent.smoothed_losses == [4.0] * 5
    for L in g["losses"]:                      # iterations 1..5; the 5th one (m = 5) decides again
        agent.step(L, g["cost_ms"][0] / 5)
    assert agent.smoothed_losses == g["smoothed"]
    assert agent.decisions == 2
    assert abs(agent.last_reward - g["reward"][0]) < 1e-12


def test_paper_defaults():
    agent = mqgrad.Mdp()
    c = agent.cfg
    assert (c.bits_min, c.bits_max, c.window, c.decide_every, c.hidden) == (2, 8, 5, 5, 10)
    assert (c.alpha, c.epsilon, c.eta, c.reward_scale) == (0.01, 0.1, 0.1, 300.0)


def test_invalid_configurations_are_rejected():
    for bad in (dict(bits_min=0), dict(bits_max=9), dict(bits_min=5, bits_max=4), dict(window=1),
                dict(decide_every=0), dict(hidden=0)):
        with pytest.raises(ValueError):
            mqgrad.Mdp(**bad)


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_bits_follow_the_papers_rules(seed):
    # widths stay in range, change only when m % T == 0, n_t never decreases, and the announced
    # width is n_t or n_t + 1 (Actions; Transition; Algorithm 2, last line)
    agent = mqgrad.Mdp(seed=seed, epsilon=0.3)
    losses = workloads.synthetic_loss_sequence(400, seed=seed)
    prev_bits, prev_n = None, 0
    for m, L in enumerate(losses):
        bits = agent.step(L, 10.0 + bits_cost(prev_bits))
        n = agent.current_bits
        assert 2 <= n <= 8 and n >= prev_n
        assert bits in (n, n + 1) and bits <= 8
        if m % 5 != 0:
            assert bits == prev_bits
        prev_bits, prev_n = bits, n
    assert agent.decisions == 80


def bits_cost(bits):
    return 0.0 if bits is None else 3.0 * bits


@pytest.mark.parametrize("cfg", [dict(seed=0), dict(seed=5, epsilon=0.3), dict(seed=9, bits_min=1, decide_every=1),
                                 dict(seed=2, bits_min=1, bits_max=8, window=4, hidden=6, alpha=0.2, discount=0.5)])
def test_library_agent_matches_the_numpy_restatement(cfg):
    lib = mqgrad.Mdp(**cfg)
    ref = mdp_ref.MdpRef(**cfg)
    losses = workloads.synthetic_loss_sequence(300, seed=cfg["seed"])
    b_lib = b_ref = None
    for m, L in enumerate(losses):
        cost = 5.0 + bits_cost(b_lib)
        b_lib = lib.step(L, cost)
        b_ref = ref.step(L, cost)
        assert b_lib == b_ref, "bit widths diverge at iteration %d" % m
        assert lib.current_bits == ref.n_t
        assert np.allclose(lib.smoothed_losses, ref.window, rtol=1e-13, atol=0)
        assert abs(lib.last_reward - ref.last_reward) <= 1e-9 * max(1.0, abs(ref.last_reward))
    assert lib.decisions == ref.decisions


def test_width_is_capped_at_the_maximum():
    agent = mqgrad.Mdp(seed=1, bits_min=7, bits_max=8, epsilon=1.0, decide_every=1)   # always explores
    seen = [agent.step(1.0 / (m + 1), 1.0) for m in range(50)]
    assert max(seen) == 8 and min(seen) >= 7
    assert agent.current_bits <= 8


def test_step_from_worker_losses_is_step_with_their_mean():
    # Algorithm 1, ReceiveLossThenSendbits: the global loss is the mean of the workers' local losses
    import random
    rnd = random.Random(4)
    a = mqgrad.Mdp(seed=9)
    b = mqgrad.Mdp(seed=9)
    for m in range(60):
        losses = [2.0 * 0.97 ** m + rnd.gauss(0, 0.01) for _ in range(5)]
        mean = 0.0
        for v in losses:
            mean = mean + v
        mean /= len(losses)
        ka = a.step_workers(losses, 50.0)
        kb = b.step(mean, 50.0)
        assert ka == kb
    assert a.smoothed_losses == b.smoothed_losses
    assert a.step_workers([], 1.0) == 0
    a.close()
    b.close()
