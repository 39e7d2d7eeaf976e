// Host-side agent that chooses the number of quantization bits: the MDP of Section 3.3 trained
// with SARSA (Algorithm 2).  Plain C++, no GPU.
//
//   time step      one decision every `decide_every` training iterations (paper: T = 5)
//   state s_t      [n_t, the last `window` moving-averaged losses]          (States; Eq. 1)
//   actions        0 = keep the bit width, 1 = one more bit                 (Actions)
//   Q(s, a)        a small MLP on the smoothed losses: window -> hidden (ReLU) -> one linear
//                  output per bit width; Q(s, a) is the output for width n_t + a    (Section 4.1)
//   policy         epsilon-greedy                                            (Policy)
//   reward         -(1 / c) * beta * reward_scale, beta = least-squares slope of the smoothed
//                  losses against 1..window, c = wall time of the period in ms      (Reward)
//   transition     n_t = n_{t-1} + argmax_a Q(s_{t-1}, a)                    (Transition)
//   learning       v += eta [r_{t-1} + discount Q(s_t, a_t) - Q(s_{t-1}, a_{t-1})] dQ/dv   (Alg. 2)
//
// Points the paper leaves open, and what is done here: the discount of the SARSA target is not
// given (configurable; default 0.9); the network has biases and is initialised U(-0.1, 0.1) from
// a seeded SplitMix64 stream; its inputs are the smoothed losses divided by the first observed
// loss; the moving average starts from the first observed loss; the window always holds the
// last `window` smoothed losses (so a decision can be taken every iteration if asked to); at
// n_t = bits_max the action "one more bit" is not available.

#include <cmath>
#include <cstdint>
#include <new>
#include <vector>

#include "mqgrad.h"

namespace {

struct SplitMix64 {
    uint64_t state;
    uint64_t next() {
        uint64_t z = (state += 0x9E3779B97F4A7C15ull);
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    }
    double uniform01() { return (double)(next() >> 11) * (1.0 / 9007199254740992.0); }  // [0, 1)
};

}  // namespace

struct mqg_mdp {
    mqg_mdp_config cfg;
    SplitMix64 rng;
    uint32_t n_out;
    // Q network, row-major: w1[hidden][window], b1[hidden], w2[n_out][hidden], b2[n_out]
    std::vector<double> w1, b1, w2, b2;
    // smoothed-loss window, oldest first
    std::vector<double> window;
    double smooth_prev;
    double first_loss;
    bool seen_loss;
    uint64_t iteration;     // m of the next call
    uint64_t decisions;     // t of the next decision
    double period_ms;       // wall time accumulated since the last decision
    uint32_t n_t;           // bit width held in the state
    uint32_t bits_out;      // width announced for the current period: n_t + a_t
    // what SARSA needs from the previous decision
    std::vector<double> prev_input;
    uint32_t prev_n;
    uint32_t prev_action;
    uint32_t prev_greedy;
    double last_reward;

    void forward(const std::vector<double>& in, std::vector<double>& hid, std::vector<double>& out) const {
        const uint32_t H = cfg.hidden, T = cfg.window;
        hid.assign(H, 0.0);
        out.assign(n_out, 0.0);
        for (uint32_t h = 0; h < H; ++h) {
            double z = b1[h];
            for (uint32_t i = 0; i < T; ++i) z += w1[h * T + i] * in[i];
            hid[h] = z > 0.0 ? z : 0.0;
        }
        for (uint32_t o = 0; o < n_out; ++o) {
            double z = b2[o];
            for (uint32_t h = 0; h < H; ++h) z += w2[o * H + h] * hid[h];
            out[o] = z;
        }
    }

    std::vector<double> network_input() const {
        std::vector<double> in(cfg.window);
        const double norm = (first_loss != 0.0) ? first_loss : 1.0;
        for (uint32_t i = 0; i < cfg.window; ++i) in[i] = window[i] / norm;
        return in;
    }

    // least-squares slope of window[i-1] against i = 1..T
    double slope() const {
        const uint32_t T = cfg.window;
        double mi = 0.0, ml = 0.0;
        for (uint32_t i = 0; i < T; ++i) { mi += (double)(i + 1); ml += window[i]; }
        mi /= T; ml /= T;
        double num = 0.0, den = 0.0;
        for (uint32_t i = 0; i < T; ++i) {
            const double di = (double)(i + 1) - mi;
            num += di * (window[i] - ml);
            den += di * di;
        }
        return num / den;
    }

    uint32_t decide() {
        std::vector<double> hid, q;
        const std::vector<double> in = network_input();
        const bool have_prev = decisions > 0;
        // Transition: n_t follows the greedy action of the previous state (or, when asked to, the action
        // that was taken, which makes the announced width monotone)
        if (have_prev) n_t = prev_n + (cfg.follow_taken_action ? prev_action : prev_greedy);
        // Reward of the previous action, from the losses and the time of the period just ended
        double reward = 0.0;
        if (have_prev) {
            const double c = period_ms > 0.0 ? period_ms : 1.0;
            reward = -(1.0 / c) * slope() * cfg.reward_scale;
            last_reward = reward;
        }
        // Policy: epsilon-greedy over the available actions
        forward(in, hid, q);
        const bool can_grow = n_t < cfg.bits_max;
        const uint32_t i0 = n_t - cfg.bits_min;
        const uint32_t greedy = (can_grow && q[i0 + 1] > q[i0]) ? 1u : 0u;   // ties keep the width
        uint32_t action = greedy;
        const double draw = rng.uniform01();
        if (can_grow && draw < cfg.epsilon) action = 1u - greedy;
        const double q_now = q[i0 + action];
        // SARSA update of the previous state-action value
        if (have_prev) {
            std::vector<double> phid, pq;
            forward(prev_input, phid, pq);
            const uint32_t po = prev_n - cfg.bits_min + prev_action;
            const double delta = reward + cfg.discount * q_now - pq[po];
            const double step = cfg.eta * delta;
            const uint32_t H = cfg.hidden, T = cfg.window;
            // dQ/dw2[po][h] = hid[h]; dQ/db2[po] = 1; dQ/dw1[h][i] = w2[po][h] * [hid[h] > 0] * in[i]
            for (uint32_t h = 0; h < H; ++h) {
                const double back = (phid[h] > 0.0) ? w2[po * H + h] : 0.0;
                for (uint32_t i = 0; i < T; ++i) w1[h * T + i] += step * back * prev_input[i];
                b1[h] += step * back;
            }
            for (uint32_t h = 0; h < H; ++h) w2[po * H + h] += step * phid[h];
            b2[po] += step;
        }
        prev_input = in;
        prev_n = n_t;
        prev_action = action;
        prev_greedy = greedy;
        decisions += 1;
        period_ms = 0.0;
        bits_out = n_t + action;
        return bits_out;
    }
};

extern "C" {

void mqg_mdp_default_config(mqg_mdp_config* cfg) {
    if (!cfg) return;
    cfg->seed = 0;
    cfg->bits_min = 2;
    cfg->bits_max = 8;
    cfg->window = 5;
    cfg->decide_every = 5;
    cfg->hidden = 10;
    cfg->alpha = 0.01;
    cfg->epsilon = 0.1;
    cfg->eta = 0.1;
    cfg->reward_scale = 300.0;
    cfg->discount = 0.9;
    cfg->follow_taken_action = 0;
}

mqg_mdp* mqg_mdp_create(const mqg_mdp_config* cfg) {
    if (!cfg) return nullptr;
    if (cfg->bits_min < 1 || cfg->bits_max > 8 || cfg->bits_min > cfg->bits_max) return nullptr;
    if (cfg->window < 2 || cfg->window > 1024 || cfg->decide_every < 1 || cfg->hidden < 1 || cfg->hidden > 4096) return nullptr;
    mqg_mdp* m = new (std::nothrow) mqg_mdp();
    if (!m) return nullptr;
    try {
    m->cfg = *cfg;
    m->rng.state = cfg->seed;
    m->n_out = cfg->bits_max - cfg->bits_min + 1;
    const uint32_t H = cfg->hidden, T = cfg->window;
    auto init = [&](std::vector<double>& v, size_t count) {
        v.resize(count);
        for (size_t i = 0; i < count; ++i) v[i] = -0.1 + 0.2 * m->rng.uniform01();
    };
    init(m->w1, (size_t)H * T);
    init(m->b1, H);
    init(m->w2, (size_t)m->n_out * H);
    init(m->b2, m->n_out);
    m->window.assign(T, 0.0);
    m->smooth_prev = 0.0;
    m->first_loss = 0.0;
    m->seen_loss = false;
    m->iteration = 0;
    m->decisions = 0;
    m->period_ms = 0.0;
    m->n_t = cfg->bits_min;
    m->bits_out = cfg->bits_min;
    m->prev_n = cfg->bits_min;
    m->prev_action = 0;
    m->prev_greedy = 0;
    m->last_reward = 0.0;
    } catch (...) {   // allocation failure: nothing crosses the C boundary
        delete m;
        return nullptr;
    }
    return m;
}

void mqg_mdp_destroy(mqg_mdp* agent) { delete agent; }

uint32_t mqg_mdp_step(mqg_mdp* agent, double loss, double elapsed_ms) {
    if (!agent) return 0;
    mqg_mdp& m = *agent;
    if (!m.seen_loss) {
        m.seen_loss = true;
        m.first_loss = loss;
        m.smooth_prev = loss;
        for (double& v : m.window) v = loss;
    }
    // Eq. (1): exponential moving average, carried across MDP time steps
    const double smooth = m.cfg.alpha * loss + (1.0 - m.cfg.alpha) * m.smooth_prev;
    m.smooth_prev = smooth;
    for (size_t i = 0; i + 1 < m.window.size(); ++i) m.window[i] = m.window[i + 1];
    m.window.back() = smooth;
    m.period_ms += elapsed_ms;
    uint32_t bits = m.bits_out;
    if (m.iteration % m.cfg.decide_every == 0) {
        try {
            bits = m.decide();
        } catch (...) {   // allocation failure inside a decision: keep the current width
            bits = m.bits_out;
        }
    }
    m.iteration += 1;
    return bits;
}

uint32_t mqg_mdp_step_workers(mqg_mdp* agent, const double* worker_losses, uint32_t P, double elapsed_ms) {
    if (!agent || !worker_losses || P == 0u) return 0;
    double sum = 0.0;
    for (uint32_t p = 0; p < P; ++p) sum = sum + worker_losses[p];
    return mqg_mdp_step(agent, sum / (double)P, elapsed_ms);
}

uint32_t mqg_mdp_current_bits(const mqg_mdp* agent) { return agent ? agent->n_t : 0u; }

void mqg_mdp_smoothed_losses(const mqg_mdp* agent, double* out) {
    if (!agent || !out) return;
    for (size_t i = 0; i < agent->window.size(); ++i) out[i] = agent->window[i];
}

double mqg_mdp_last_reward(const mqg_mdp* agent) { return agent ? agent->last_reward : 0.0; }

uint64_t mqg_mdp_decisions(const mqg_mdp* agent) { return agent ? agent->decisions : 0u; }

// ---- the Q network's parameter vector v, laid out [W1 row by row, b1, W2 row by row, b2] ------------

uint32_t mqg_mdp_num_weights(const mqg_mdp* agent) {
    if (!agent) return 0u;
    return (uint32_t)(agent->w1.size() + agent->b1.size() + agent->w2.size() + agent->b2.size());
}

void mqg_mdp_get_weights(const mqg_mdp* agent, double* out) {
    if (!agent || !out) return;
    for (const std::vector<double>* part : {&agent->w1, &agent->b1, &agent->w2, &agent->b2}) {
        for (double x : *part) *out++ = x;
    }
}

void mqg_mdp_set_weights(mqg_mdp* agent, const double* in) {
    if (!agent || !in) return;
    for (std::vector<double>* part : {&agent->w1, &agent->b1, &agent->w2, &agent->b2}) {
        for (double& x : *part) x = *in++;
    }
}

void mqg_mdp_q_values(const mqg_mdp* agent, const double* input, double* out) {
    if (!agent || !input || !out) return;
    try {
        const std::vector<double> in(input, input + agent->cfg.window);
        std::vector<double> hid, q;
        agent->forward(in, hid, q);
        for (uint32_t o = 0; o < agent->n_out; ++o) out[o] = q[o];
    } catch (...) {   // allocation failure: nothing crosses the C boundary
    }
}

// ---- the "Adaptive" baseline's rule (Section 4.1): bits from the mean gradient norm ----------------

void mqg_adaptive_default_config(mqg_adaptive_config* cfg) {
    if (!cfg) return;
    cfg->base_bits = 2;
    cfg->norm_per_bit = 0.0005;
    cfg->bits_min = 2;
    cfg->bits_max = 8;
}

mqg_status mqg_adaptive_bits(const double* worker_norms, uint32_t W, const mqg_adaptive_config* cfg,
                             uint32_t* bits_out) {
    if (!worker_norms || !cfg || !bits_out || W == 0u) return MQG_EINVAL;
    if (!(cfg->norm_per_bit > 0.0) || cfg->bits_min < 1u || cfg->bits_max > 8u || cfg->bits_min > cfg->bits_max ||
        cfg->base_bits > 8u)
        return MQG_EINVAL;
    double z = 0.0;
    for (uint32_t w = 0; w < W; ++w) {
        if (!(worker_norms[w] >= 0.0)) return MQG_EINVAL;   // negative or NaN
        z = z + worker_norms[w];
    }
    z = z / (double)W;
    uint32_t k = cfg->bits_max;
    if (std::isfinite(z)) {
        const double extra = std::floor(z / cfg->norm_per_bit);
        if (extra < 16.0) k = cfg->base_bits + (uint32_t)extra;
    }
    if (k < cfg->bits_min) k = cfg->bits_min;
    if (k > cfg->bits_max) k = cfg->bits_max;
    *bits_out = k;
    return MQG_OK;
}

}  // extern "C"
