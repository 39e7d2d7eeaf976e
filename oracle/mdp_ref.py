"""The paper's bit-width agent written out from Section 3.3 and Algorithm 2 (MQGrad-SARSA) in plain
Python/numpy -- test infrastructure, not product code.

The agent is a set of functions named as the paper names them, over one flat parameter vector v:

  q_function(v, shape, L)          Q network (Section 4.1): L = the T smoothed losses (States, Eq. 1) ->
                                   hidden ReLU units -> one linear output per bit width; Q(s, a) is the
                                   output that belongs to width n + a
  q_gradient(v, shape, L, o)       dQ_o/dv, the factor of Algorithm 2's update, by the chain rule
  transition(n, greedy_action)     Transition: n_t = n_{t-1} + argmax_a Q(s_{t-1}, a)
  reward(Lbar, c, gamma)           Reward: -(1/c) * beta * gamma, beta = least-squares slope of Lbar on 1..T
  policy(q, n, ...)                Policy: epsilon-greedy over {0: keep, 1: one more bit}
  moving_average(...)              Eq. (1)

and `MdpRef.step` strings them together in the order of Algorithm 2: s_t <- T(s_{t-1}, a_{t-1});
r_{t-1} <- R; a_t ~ pi(s_t); v <- v + eta [r_{t-1} + discount * Q(s_t, a_t) - Q(s_{t-1}, a_{t-1})] dQ/dv
evaluated at (s_{t-1}, a_{t-1}); return n_t + a_t.

Where the paper is silent this file takes the readings listed in the design notes: the SARSA discount is a
parameter (default 0.9; the paper gives no value, so the learning dynamics are not fixed by it -- the update
itself is pinned by a hand-computed step and by finite differences in tests/test_mdp.py); the network has
biases; v starts ~ U(-0.1, 0.1) from a seeded SplitMix64 stream in the order [W1 row by row, b1, W2 row by
row, b2] (both sides implement that generator, which also supplies the epsilon-greedy draws); the inputs
are the smoothed losses divided by the first loss; the moving average starts at the first loss; the window
of T smoothed losses slides every iteration; "one more bit" does not exist at the maximum width.
"""
import numpy as np

MASK64 = (1 << 64) - 1


class SplitMix64:
    """Steele, Lea & Flood's SplitMix64: the published constants, 53-bit uniforms in [0, 1)."""

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


def reward(smoothed, cost_ms, gamma):
    """Reward: R = -(1 / c) * beta * gamma."""
    return -(1.0 / cost_ms) * slope(smoothed) * gamma


def transition(n_prev, greedy_prev):
    """Transition: the state's width moves by the greedy action of the previous state."""
    return n_prev + greedy_prev


def unpack(v, shape):
    """Views of the flat parameter vector: W1 (H x T), b1 (H), W2 (O x H), b2 (O)."""
    T, H, O = shape
    i = 0
    W1 = v[i:i + H * T].reshape(H, T); i += H * T
    b1 = v[i:i + H]; i += H
    W2 = v[i:i + O * H].reshape(O, H); i += O * H
    b2 = v[i:i + O]
    return W1, b1, W2, b2


def q_function(v, shape, L):
    """All outputs of the Q network for input L: W2 relu(W1 L + b1) + b2."""
    W1, b1, W2, b2 = unpack(v, shape)
    return W2 @ np.maximum(W1 @ L + b1, 0.0) + b2


def q_gradient(v, shape, L, o):
    """dQ_o/dv as a flat vector laid out like v.  With z = W1 L + b1 and h = relu(z):
    dQ_o/dW2[o] = h, dQ_o/db2[o] = 1, dQ_o/db1 = W2[o] * [z > 0], dQ_o/dW1 = outer(dQ_o/db1, L);
    the rows of W2 and entries of b2 of the other outputs get 0."""
    T, H, O = shape
    W1, b1, W2, b2 = unpack(v, shape)
    z = W1 @ L + b1
    g = np.zeros_like(v)
    gW1, gb1, gW2, gb2 = unpack(g, shape)
    gb1[:] = W2[o] * (z > 0.0)
    gW1[:, :] = np.outer(gb1, L)
    gW2[o, :] = np.maximum(z, 0.0)
    gb2[o] = 1.0
    return g


def policy(q, n, bits_min, bits_max, epsilon, draw):
    """epsilon-greedy over the available actions; returns (taken action, greedy action).  Ties keep the
    width (the paper keeps n when Q(s, 0) >= Q(s, 1))."""
    if n >= bits_max:
        return 0, 0
    greedy = 1 if q[n - bits_min + 1] > q[n - bits_min] else 0
    return (1 - greedy if draw < epsilon else greedy), greedy


class MdpRef:
    def __init__(self, seed=0, bits_min=2, bits_max=8, window=5, decide_every=5, hidden=10,
                 alpha=0.01, epsilon=0.1, eta=0.1, reward_scale=300.0, discount=0.9, follow_taken_action=0):
        self.bits_min, self.bits_max = bits_min, bits_max
        self.T, self.decide_every = window, decide_every
        self.alpha, self.epsilon, self.eta = alpha, epsilon, eta
        self.reward_scale, self.discount = reward_scale, discount
        self.follow_taken_action = follow_taken_action
        self.shape = (window, hidden, bits_max - bits_min + 1)
        self.rng = SplitMix64(seed)
        count = hidden * window + hidden + self.shape[2] * hidden + self.shape[2]
        self.v = np.array([-0.1 + 0.2 * self.rng.uniform01() for _ in range(count)])
        self.window = None          # the T most recent smoothed losses, oldest first
        self.smooth_prev = None
        self.first_loss = None
        self.iteration = 0
        self.decisions = 0
        self.period_ms = 0.0
        self.n_t = bits_min
        self.bits_out = bits_min
        self.last = None            # (L, n, a, greedy a) of time step t - 1
        self.last_reward = 0.0

    def state_input(self):
        norm = self.first_loss if self.first_loss != 0.0 else 1.0
        return np.array(self.window) / norm

    def sarsa(self):
        """One MDP time step: the five lines of Algorithm 2."""
        L_t = self.state_input()
        r_prev = None
        if self.last is not None:
            L_prev, n_prev, a_prev, greedy_prev = self.last
            self.n_t = transition(n_prev, a_prev if self.follow_taken_action else greedy_prev)      # line 1
            r_prev = reward(self.window, self.period_ms if self.period_ms > 0.0 else 1.0, self.reward_scale)   # line 2
            self.last_reward = r_prev
        q_t = q_function(self.v, self.shape, L_t)
        draw = self.rng.uniform01()
        a_t, greedy_t = policy(q_t, self.n_t, self.bits_min, self.bits_max, self.epsilon, draw)      # line 3
        if self.last is not None:                                                                    # line 4
            o_prev = n_prev - self.bits_min + a_prev
            o_t = self.n_t - self.bits_min + a_t
            q_prev = q_function(self.v, self.shape, L_prev)[o_prev]
            td = r_prev + self.discount * q_t[o_t] - q_prev
            self.v = self.v + self.eta * td * q_gradient(self.v, self.shape, L_prev, o_prev)
        self.last = (L_t, self.n_t, a_t, greedy_t)
        self.decisions += 1
        self.period_ms = 0.0
        self.bits_out = self.n_t + a_t                                                               # line 5
        return self.bits_out

    def step(self, loss, elapsed_ms):
        """One training iteration m: smooth the loss (Eq. 1), and when m is a multiple of `decide_every`
        run one MDP time step; otherwise the previous width is sent again."""
        if self.window is None:
            self.first_loss = loss
            self.smooth_prev = loss
            self.window = [loss] * self.T
        self.smooth_prev = moving_average([loss], self.alpha, self.smooth_prev)[0]
        self.window = self.window[1:] + [self.smooth_prev]
        self.period_ms += elapsed_ms
        bits = self.bits_out
        if self.iteration % self.decide_every == 0:
            bits = self.sarsa()
        self.iteration += 1
        return bits
