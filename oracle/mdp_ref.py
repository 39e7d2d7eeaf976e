"""The paper's bit-width agent restated in plain Python/numpy -- test infrastructure, not product code.

Follows Section 3.3 and Algorithm 2 (MQGrad-SARSA) of the paper step by step:

  time step     one decision every `decide_every` training iterations (the paper's T = 5)
  state         s_t = [n_t, Lbar_t], Lbar_t the last `window` moving-averaged losses      (States, Eq. 1)
  actions       0 keeps the width, 1 adds one bit; widths never decrease                    (Actions)
  Q function    MLP: window inputs -> hidden ReLU units -> one linear output per bit width;
                Q(s, a) is the output for width n_t + a                                      (Q function, Section 4.1)
  policy        epsilon-greedy                                                               (Policy)
  reward        R = -(1 / c) * beta * reward_scale, beta the least-squares slope of the
                smoothed losses against i = 1..window, c the period's wall time in ms       (Reward)
  transition    n_t = n_{t-1} + argmax_a Q(s_{t-1}, a)                                       (Transition)
  learning      v <- v + eta [r_{t-1} + discount * Q(s_t, a_t) - Q(s_{t-1}, a_{t-1})] dQ/dv  (Algorithm 2)

Where the paper is silent this file takes the same readings as the library (they are listed in the
design notes): SARSA discount configurable (default 0.9, the paper gives no value: parity of the
learning dynamics is unpinned), biases in the network, weights ~ U(-0.1, 0.1) from a seeded
SplitMix64 stream (each side implements the same generator), inputs divided by the first loss,
the moving average starts at the first loss, the window slides every iteration, and "one more bit"
is unavailable at the maximum width.
"""
import numpy as np

MASK64 = (1 << 64) - 1


class SplitMix64:
    def __init__(self, seed):
        self.state = seed & MASK64

    def next(self):
        self.state = (self.state + 0x9E3779B97F4A7C15) & MASK64
        z = self.state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK64
        return z ^ (z >> 31)

    def uniform01(self):
        return (self.next() >> 11) * (1.0 / 9007199254740992.0)


def moving_average(losses, alpha, start):
    """Eq. (1): Lbar^i = alpha * L^i + (1 - alpha) * Lbar^{i-1}, carried across time steps."""
    out, prev = [], start
    for L in losses:
        prev = alpha * L + (1.0 - alpha) * prev
        out.append(prev)
    return out


def slope(values):
    """beta of  argmin_{beta, b} sum_i (beta * i + b - values[i-1])^2,  i = 1..T  (Reward)."""
    T = len(values)
    i = np.arange(1, T + 1, dtype=np.float64)
    A = np.stack([i, np.ones(T)], axis=1)
    beta, _ = np.linalg.lstsq(A, np.asarray(values, dtype=np.float64), rcond=None)[0]
    return float(beta)


class MdpRef:
    def __init__(self, seed=0, bits_min=2, bits_max=8, window=5, decide_every=5, hidden=10,
                 alpha=0.01, epsilon=0.1, eta=0.1, reward_scale=300.0, discount=0.9):
        self.bits_min, self.bits_max = bits_min, bits_max
        self.window_len, self.decide_every, self.hidden = window, decide_every, hidden
        self.alpha, self.epsilon, self.eta = alpha, epsilon, eta
        self.reward_scale, self.discount = reward_scale, discount
        self.rng = SplitMix64(seed)
        self.n_out = bits_max - bits_min + 1
        u = lambda count: np.array([-0.1 + 0.2 * self.rng.uniform01() for _ in range(count)])
        self.w1 = u(hidden * window).reshape(hidden, window)
        self.b1 = u(hidden)
        self.w2 = u(self.n_out * hidden).reshape(self.n_out, hidden)
        self.b2 = u(self.n_out)
        self.window = None
        self.smooth_prev = None
        self.first_loss = None
        self.iteration = 0
        self.decisions = 0
        self.period_ms = 0.0
        self.n_t = bits_min
        self.bits_out = bits_min
        self.prev = None          # (input, n, action, greedy) of the previous decision
        self.last_reward = 0.0

    def q_values(self, x):
        hid = np.maximum(self.w1 @ x + self.b1, 0.0)
        return hid, self.w2 @ hid + self.b2

    def _decide(self):
        norm = self.first_loss if self.first_loss != 0.0 else 1.0
        x = np.array(self.window) / norm
        if self.prev is not None:
            p_in, p_n, p_action, p_greedy = self.prev
            self.n_t = p_n + p_greedy                                   # Transition
            c = self.period_ms if self.period_ms > 0.0 else 1.0
            reward = -(1.0 / c) * slope(self.window) * self.reward_scale   # Reward
            self.last_reward = reward
        hid, q = self.q_values(x)
        can_grow = self.n_t < self.bits_max
        i0 = self.n_t - self.bits_min
        greedy = 1 if (can_grow and q[i0 + 1] > q[i0]) else 0
        action = greedy
        draw = self.rng.uniform01()
        if can_grow and draw < self.epsilon:                             # Policy: epsilon-greedy
            action = 1 - greedy
        q_now = q[i0 + action]
        if self.prev is not None:                                        # Algorithm 2: SARSA update
            p_hid, p_q = self.q_values(p_in)
            po = p_n - self.bits_min + p_action
            delta = reward + self.discount * q_now - p_q[po]
            step = self.eta * delta
            back = np.where(p_hid > 0.0, self.w2[po], 0.0)
            self.w1 += step * np.outer(back, p_in)
            self.b1 += step * back
            self.w2[po] += step * p_hid
            self.b2[po] += step
        self.prev = (x, self.n_t, action, greedy)
        self.decisions += 1
        self.period_ms = 0.0
        self.bits_out = self.n_t + action
        return self.bits_out

    def step(self, loss, elapsed_ms):
        if self.window is None:
            self.first_loss = loss
            self.smooth_prev = loss
            self.window = [loss] * self.window_len
        smooth = self.alpha * loss + (1.0 - self.alpha) * self.smooth_prev   # Eq. (1)
        self.smooth_prev = smooth
        self.window = self.window[1:] + [smooth]
        self.period_ms += elapsed_ms
        bits = self.bits_out
        if self.iteration % self.decide_every == 0:
            bits = self._decide()
        self.iteration += 1
        return bits
