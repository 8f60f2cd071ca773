// HALoS server-side update rules -- plain CPU oracle.
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, single-threaded,
// obviously-correct statement of what the local parameter servers (LPS) and
// the global parameter server (GPS) compute.  It exists so that the GPU
// library can be checked against something written independently from the
// paper; it shares no code, header, table or helper with that library and
// nothing in the product path may call it.
//
// What it follows (HALoS, arXiv 2506.04531):
//   * Algorithm 1 "HALoS Update Rules": the GPS block (receive Delta, update,
//     send the model back), the LPS block (update on every worker delta, send
//     Delta = theta_t - theta_{t_last} after K updates, merge the returned
//     global model with weight alpha and reset t_last).
//   * Sec. 4.1 item 2: worker deltas and returned global models share ONE
//     queue per LPS and are handled in arrival order.
//   * Appendix E, first two displays: ModelUpdate is
//         m  <- beta * m + grad
//         x  <- x - eta * [ (1 - beta) * grad + beta * m ]
//     for both tiers.  "grad" is the pseudo-gradient, i.e. the NEGATIVE of the
//     delta that Algorithm 1 sends (delta = end - start model), so that
//     beta = 0, eta = 1 adopts the sender's progress:  x <- x + delta.
//
// Readings taken where the paper is silent (each is listed in the design
// document of this repository):
//   * The coefficient on grad is kept as a parameter cg; the paper's value is
//     cg = 1 - beta.  cg = 1 gives the textbook Nesterov step.
//   * theta_{t_last} is the model right AFTER the merge (the merge branch first sets t_last,
//     then overwrites theta_t), so updates applied while a Delta is in
//     flight are never part of any later Delta.
//   * At most one Delta per LPS is in flight: the send test is
//     "t - t_last >= K and nothing in flight", which equals the paper's
//     "t - t_last = K" whenever K only changes at a merge.
//   * The model the LPS merges is the GPS model right after THAT LPS's Delta
//     was applied, even if other LPSs update the GPS before it is merged.
//   * Delta is applied at the GPS unnormalised (no 1/K, no 1/M).
//
// Delayed Nesterov momentum (optional, per tier).  The paper's runs use, at both tiers, the delayed
// Nesterov optimizer of the Async-Local-SGD work it cites (Sec. 5.1; App. D lists the delays d_l, d_g and
// gives the listed rates as eta / d), but does not restate it.  The rule implemented here is that published algorithm with its default momentum activation of
// zero, carried over to this paper's ModelUpdate by keeping the coefficient cg on the gradient term:
//     every update:        buffer <- buffer + grad;  x <- x - eta * (cg / d) * grad
//     every d-th update:   m <- beta * m + buffer / d;  x <- x - eta * [ (cg / d) * grad + beta * m ];
//                          buffer <- 0
// With d = 1 every update is a "d-th" one and the rule is exactly ModelUpdate above.  The buffer and the
// position in the cycle belong to the server; merges do not touch them.
//
// Comparison rules on the same servers (Sec. 2 and the ablation of Sec. 5.2 name them; each is a small variation
// of the steps above, stated here in this file's own terms):
//   * weighted arrival: a delta may carry a scalar weight w chosen by the caller (a staleness-scaled update as in
//     the asynchronous-federated baseline of Sec. 5.2; the paper names only the polynomial's exponent, so the
//     weight's formula stays outside); the server applies ModelUpdate to w * grad.  w = 1 changes nothing.
//   * averaged step: the n deltas at the head of the queue are averaged, (g_1 + ... + g_n) * (1/n) summed in
//     arrival order, and applied as ONE update (the synchronous outer step of the Local-SGD methods in Sec. 2).
//   * single tier: the global server applies a worker's delta itself with its own rule (no local server;
//     App. D lists this baseline's hyper-parameters), gps_apply_delta below.
// Deltas may also arrive as IEEE half precision (the workers of Sec. 5.1 train in fp16): upcast exactly.
//
// Momentum kept in bfloat16 (an option of this repository, not of the paper, which does not state the servers'
// precision): after  m <- beta * m + grad  the new momentum is rounded to bfloat16 (round to nearest, ties to
// even, decided on the binary32 value) and it is that rounded value which enters the step and is carried over.
// Model, accumulated update and returned global model stay in full precision.  Not combined with the delayed rule.
// Pins (tests/test_oracle_variants.py): the rounding against torch's conversion, hand-computed ties, equality
// with full-precision momentum whenever nothing needs rounding.
//
// Two numerical forms are provided and selected at creation:
//   form 0 (literal)      keeps the snapshot theta_{t_last} and forms Delta by
//                         subtraction exactly as Algorithm 1's LPS block writes it;
//   form 1 (accumulator)  keeps a running sum of the applied steps instead.
// In exact arithmetic they are the same; in fp64 they agree to ~1e-13.
// Precision is fp64 (the reference) or fp32 (same operation order as a
// single-pass fp32 implementation would use; useful as a bit-level check).
//
// Pins (tests/test_oracle_pins.py): local-SGD special case, K identical deltas,
// geometric momentum series, IIR-filter closed form via scipy.signal.lfilter,
// torch.optim.SGD(nesterov) for cg = 1, the theta - eta (g + beta^2 m_old)
// identity from the proof, merge endpoints alpha in {0, 1}, geometric
// contraction of repeated merges, hierarchy collapse to one level, linearity,
// snapshot == accumulator, bf16 upcast vs torch, protocol counters.
// Delayed momentum has its own pins (tests/test_oracle_delayed_momentum.py): d = 1 equals the plain rule bit
// for bit, beta = 0 is SGD at rate eta / d (the paper's statement about the rule), momentum as a filter over
// cycle means, a constant-delta closed form, merges leave the cycle alone.  Its DEFINITION, though, is the cited
// work's, not this paper's: on that count parity unpinned.
// Full-size end states (hundreds of events on 70M..1B parameters) have no
// external reference: they are pinned only through the tiny cases above plus
// elementwise independence -- otherwise parity unpinned.

#include <chrono>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <deque>
#include <vector>

namespace {

enum ItemKind { ITEM_DELTA = 1, ITEM_GLOBAL = 2 };
enum Phase {
    ACCUMULATING = 0,   // no Delta in flight
    SENT = 1,           // Delta frozen and travelling to the GPS
    RETURNING = 2,      // GPS has applied it; the global model is travelling back
    QUEUED = 3          // the global model sits in this LPS's queue
};

struct StepInfo {       // what one lps_step did (mirrors nothing: its own layout)
    int32_t kind;       // 0 nothing queued, 1 worker update, 2 global-model merge
    int32_t sent;       // 1 if this update reached the accumulation count and froze a Delta
    int32_t accumulated;// 1 if this update counted towards the Delta being accumulated
    int32_t worker;     // worker whose delta was applied (-1 for a merge)
    int64_t t;
    int64_t t_last;
};

template <class R>
struct Rule { R eta, beta, cg; };

// ModelUpdate (Appendix E): momentum first, then the step.  Returns the step
// that was subtracted so that callers can accumulate it.
// binary32 -> bfloat16 bit pattern: round to nearest, ties to even; any NaN becomes the quiet NaN 0x7FC0.
inline uint16_t f32_to_bf16(float f) {
    uint32_t u;
    std::memcpy(&u, &f, sizeof u);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0u;
    u += 0x7FFFu + ((u >> 16) & 1u);                     // half an ulp, less one bit when the kept part is even
    return (uint16_t)(u >> 16);
}

inline float bf16_value(uint16_t bits) {                 // bfloat16 is the upper half of a binary32
    uint32_t u = (uint32_t)bits << 16;
    float f;
    std::memcpy(&f, &u, sizeof f);
    return f;
}

template <class R>
inline R model_update(R &x, R &m, R grad, const Rule<R> &r, bool m_bf16 = false) {
    m = std::fma(r.beta, m, grad);                       // m <- beta m + grad
    if (m_bf16) m = R(bf16_value(f32_to_bf16((float)m)));   // momentum kept in bfloat16: the rounded value is the state
    R direction = std::fma(r.beta, m, r.cg * grad);      // (1-beta) grad + beta m   (cg = 1-beta)
    R step = r.eta * direction;
    x = x - step;
    return step;
}

// Delayed Nesterov momentum: one server's position in its cycle of d updates.
template <class R>
struct Delay {
    bool enabled = false;   // false: plain ModelUpdate (the default); true: the delayed rule, also for d = 1
    int32_t d = 1;
    int32_t seen = 0;       // updates applied since the last momentum refresh, 0 .. d-1
    R inv_d = R(1);         // 1 / d
    void set(int32_t d_) { enabled = true; d = d_; seen = 0; inv_d = R(1) / R(d_); }
};

// One element of the delayed rule.  `first`: this update opens a cycle (the buffer holds nothing yet);
// `refresh`: it closes one (momentum is refreshed from the cycle's mean gradient and applied).
template <class R>
inline R delayed_update(R &x, R &m, R &buffer, R grad, const Rule<R> &r, R inv_d, bool first, bool refresh) {
    buffer = first ? grad : buffer + grad;               // sum of the cycle's gradients so far
    const R grad_part = (r.cg * inv_d) * grad;           // the rate on the gradient is divided by d
    R direction = grad_part;
    if (refresh) {
        m = std::fma(r.beta, m, buffer * inv_d);         // m <- beta m + mean gradient of the cycle
        direction = std::fma(r.beta, m, grad_part);
        buffer = R(0);
    }
    R applied = r.eta * direction;
    x = x - applied;
    return applied;
}

// Error-scale bookkeeping (not part of the algorithm).  A reduced-precision implementation's error
// in an element is proportional to the largest magnitudes that ever flowed into it, not to its current
// value: momentum that has cancelled down to almost nothing still carries the rounding error of its
// former size, and a step whose two terms cancel is tiny while its rounding error is not.  So every
// array carries, per element, a scale that is propagated like the values themselves but with absolute
// values and max instead of signed sums:
//     scale(m)    >= |grad|, |m|                              (and it never shrinks)
//     step scale   = |eta| (|cg| |grad scale| + |beta| scale(m))
//     scale(x)    >= step scale, |x|        for the model and for the accumulated update
// and a merge or a hand-over copies the source's scale along with its values.
template <class R>
inline R step_scale(R m_scale, R grad_scale, const Rule<R> &r) {
    return std::fabs(r.eta) * (std::fabs(r.cg) * grad_scale + std::fabs(r.beta) * m_scale);
}

template <class R>
inline void raise_to(R &scale, R v) { if (v > scale) scale = v; }

// The same bookkeeping for the delayed rule: the buffer's scale is the sum of the magnitudes added to it, the
// momentum's scale rises to the mean it absorbs at a refresh; returns the step's scale.
template <class R>
inline R delayed_scales(R &m_scale, R &buffer_scale, R m_now, R grad, const Rule<R> &r, R inv_d, bool first, bool refresh) {
    const R g_mag = std::fabs(grad);
    buffer_scale = first ? g_mag : buffer_scale + g_mag;
    R terms = std::fabs(r.eta) * std::fabs(r.cg) * inv_d * g_mag;
    if (refresh) {
        raise_to(m_scale, buffer_scale * inv_d);
        raise_to(m_scale, std::fabs(m_now));
        terms += std::fabs(r.eta) * std::fabs(r.beta) * m_scale;
    }
    return terms;
}

template <class R>
struct QueueItem {
    int kind;
    int worker;
    std::vector<float> grad;     // pseudo-gradient values (exactly representable in fp32)
    float weight = 1.0f;         // caller's scalar on this delta (1 = plain arrival)
};

template <class R>
struct Lps {
    std::vector<R> theta, m;
    std::vector<R> snap;         // form 0: theta_{t_last}
    std::vector<R> acc;          // form 1: sum of steps since t_last
    std::vector<R> frozen;       // G = theta_{t_last} - theta_t at the send (= -Delta)
    std::vector<R> inbox;        // the global model returned for this LPS
    std::vector<R> sc_theta, sc_m, sc_aux;   // error scales, see step_scale()
    Delay<R> delay;              // delayed Nesterov momentum of this server
    std::vector<R> buffer, sc_buffer;        // its gradient buffer (sum over the open cycle) and error scale
    std::deque<QueueItem<R>> queue;
    std::vector<char> worker_queued;
    int64_t t = 0, t_last = 0;
    int32_t K = 1;
    int phase = ACCUMULATING;
    // monitors (Sec. 4.2, assumptions 4 and 5): squared norm of the last applied delta, squared distance between
    // the local model and the global model at the last merge (before merging).  Plain fp64 sums.
    double last_delta_sq = 0.0, last_merge_dist_sq = 0.0;
};

template <class R>
struct Oracle {
    int64_t n;
    int form;
    Rule<R> local, global;
    R alpha;
    std::vector<R> Theta, M, sc_Theta, sc_M;
    bool momentum_bf16 = false;     // every server's momentum is rounded to bfloat16 whenever it is updated
    Delay<R> gps_delay;
    std::vector<R> gps_buffer, sc_gps_buffer;
    int64_t gps_updates = 0;
    std::vector<Lps<R>> lps;
    // Stopwatch (not part of the algorithm): seconds spent inside, and calls of, the three event handlers, so that a
    // benchmark can quote this code's own speed per event type without the cost of getting data to it.
    double seconds[3] = {0.0, 0.0, 0.0};     // 0 worker update, 1 GPS update, 2 merge
    int64_t calls[3] = {0, 0, 0};
    struct Stopwatch {
        double &acc; int64_t &n; std::chrono::steady_clock::time_point t0;
        Stopwatch(double &a, int64_t &c) : acc(a), n(c), t0(std::chrono::steady_clock::now()) {}
        ~Stopwatch() { acc += std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count(); n += 1; }
    };

    static void grow(std::vector<R> &scale, const std::vector<R> &v) {
        for (size_t j = 0; j < v.size(); ++j) {
            R a = std::fabs(v[j]);
            if (a > scale[j]) scale[j] = a;
        }
    }

    Oracle(int64_t n_, int n_lps, int form_, Rule<R> loc, Rule<R> glob, R alpha_,
           const int32_t *K, const float *theta0)
        : n(n_), form(form_), local(loc), global(glob), alpha(alpha_) {
        Theta.assign(theta0, theta0 + n);
        M.assign(n, R(0));
        sc_Theta.assign(n, R(0)); sc_M.assign(n, R(0));
        gps_buffer.assign(n, R(0)); sc_gps_buffer.assign(n, R(0));
        grow(sc_Theta, Theta);
        lps.resize(n_lps);
        for (int l = 0; l < n_lps; ++l) {
            Lps<R> &s = lps[l];
            s.theta = Theta;                 // LPS initialisation: theta_0 <- Theta_0
            s.m.assign(n, R(0));
            s.snap = Theta;
            s.acc.assign(n, R(0));
            s.frozen.assign(n, R(0));
            s.inbox.assign(n, R(0));
            s.sc_theta.assign(n, R(0)); s.sc_m.assign(n, R(0)); s.sc_aux.assign(n, R(0));
            s.buffer.assign(n, R(0)); s.sc_buffer.assign(n, R(0));
            grow(s.sc_theta, s.theta);
            s.K = K[l];
        }
    }

    // LPS block, "receive delta": a worker's delta arrives and joins the queue.
    int arrive_delta(int l, int worker, const float *g, float weight = 1.0f) {
        Lps<R> &s = lps[l];
        if (worker < 0) return -1;
        if ((size_t)worker >= s.worker_queued.size()) s.worker_queued.resize(worker + 1, 0);
        if (s.worker_queued[worker]) return -2;            // one delta per worker at a time
        s.worker_queued[worker] = 1;
        QueueItem<R> it;
        it.kind = ITEM_DELTA; it.worker = worker; it.grad.assign(g, g + n); it.weight = weight;
        s.queue.push_back(std::move(it));
        return 0;
    }

    // LPS block, "receive Theta_i": the global model sent back by the GPS arrives and joins the same queue.
    int arrive_global(int l) {
        Lps<R> &s = lps[l];
        if (s.phase != RETURNING) return -2;
        s.phase = QUEUED;
        QueueItem<R> it; it.kind = ITEM_GLOBAL; it.worker = -1;
        s.queue.push_back(std::move(it));
        return 0;
    }

    // One worker update of server s with the pseudo-gradient gvec (already weighted or averaged): the counter, ModelUpdate,
    // the accumulation and the send test of the LPS block.
    void apply_update(Lps<R> &s, const std::vector<R> &gvec, StepInfo &out) {
        Stopwatch watch(seconds[0], calls[0]);
        s.t += 1;                                                       // t <- t + 1
        const bool accumulate = (s.phase == ACCUMULATING);
        s.last_delta_sq = 0.0;
        for (int64_t j = 0; j < n; ++j) s.last_delta_sq += (double)gvec[j] * (double)gvec[j];
        const bool first = s.delay.seen == 0, refresh = s.delay.seen + 1 == s.delay.d;
        for (int64_t j = 0; j < n; ++j) {                               // ModelUpdate
            const R grad = gvec[j];
            R step, terms;
            if (s.delay.enabled) {
                step = delayed_update<R>(s.theta[j], s.m[j], s.buffer[j], grad, local, s.delay.inv_d, first, refresh);
                terms = delayed_scales<R>(s.sc_m[j], s.sc_buffer[j], s.m[j], grad, local, s.delay.inv_d, first, refresh);
            } else {
                step = model_update<R>(s.theta[j], s.m[j], grad, local, momentum_bf16);
                raise_to(s.sc_m[j], std::fabs(grad));
                raise_to(s.sc_m[j], std::fabs(s.m[j]));
                terms = step_scale<R>(s.sc_m[j], std::fabs(grad), local);
            }
            if (form == 1 && accumulate) s.acc[j] = s.acc[j] + step;
            raise_to(s.sc_theta[j], terms);
            raise_to(s.sc_theta[j], std::fabs(s.theta[j]));
            if (accumulate) {
                raise_to(s.sc_aux[j], terms);
                raise_to(s.sc_aux[j], std::fabs(form == 1 ? s.acc[j] : s.snap[j] - s.theta[j]));
            }
        }
        if (s.delay.enabled) s.delay.seen = refresh ? 0 : s.delay.seen + 1;
        out.kind = 1; out.accumulated = accumulate ? 1 : 0;
        if (accumulate && s.t - s.t_last >= s.K) {                      // send test
            for (int64_t j = 0; j < n; ++j)                             // Delta, sign flipped: G = -Delta
                s.frozen[j] = (form == 1) ? s.acc[j] : (s.snap[j] - s.theta[j]);
            s.phase = SENT;
            out.sent = 1;
        }
    }

    // Averaged step: the `count` deltas at the head of the queue become ONE update with their mean,
    // (w_1 g_1 + ... + w_n g_n) * (1/n), added up in arrival order.  count = 1 is the plain update.
    int lps_step_average(int l, int count, StepInfo *info) {
        Lps<R> &s = lps[l];
        if (count < 1 || (size_t)count > s.queue.size()) return -2;
        for (int i = 0; i < count; ++i) if (s.queue[i].kind != ITEM_DELTA) return -2;
        StepInfo out{}; out.worker = -1;
        std::vector<R> gvec(n);
        for (int i = 0; i < count; ++i) {
            QueueItem<R> it = std::move(s.queue.front());
            s.queue.pop_front();
            const R w = R(it.weight);
            for (int64_t j = 0; j < n; ++j) {
                const R term = w * R(it.grad[j]);
                gvec[j] = (i == 0) ? term : gvec[j] + term;
            }
            s.worker_queued[it.worker] = 0;
            out.worker = it.worker;
        }
        const R inv_n = R(1) / R(count);
        for (int64_t j = 0; j < n; ++j) gvec[j] = gvec[j] * inv_n;
        apply_update(s, gvec, out);
        out.t = s.t; out.t_last = s.t_last;
        *info = out;
        return 0;
    }

    // Handle the head of the queue: the update branch for a delta, the merge branch for a global model.
    int lps_step(int l, StepInfo *info) {
        Lps<R> &s = lps[l];
        StepInfo out{}; out.worker = -1;
        if (s.queue.empty()) { out.t = s.t; out.t_last = s.t_last; *info = out; return 0; }
        QueueItem<R> it = std::move(s.queue.front());
        s.queue.pop_front();
        if (it.kind == ITEM_DELTA) {
            std::vector<R> gvec(n);
            const R w = R(it.weight);                                   // the caller's scalar on this delta (1 = none)
            for (int64_t j = 0; j < n; ++j) gvec[j] = w * R(it.grad[j]);
            apply_update(s, gvec, out);
            s.worker_queued[it.worker] = 0;
            out.worker = it.worker;
        } else {
            if (s.phase != QUEUED) return -3;
            Stopwatch watch(seconds[2], calls[2]);
            s.t_last = s.t;                                             // t_last <- t
            const R keep = R(1) - alpha;
            s.last_merge_dist_sq = 0.0;
            for (int64_t j = 0; j < n; ++j) {
                const double d = (double)s.theta[j] - (double)s.inbox[j];
                s.last_merge_dist_sq += d * d;
            }
            for (int64_t j = 0; j < n; ++j) {                           // merge
                raise_to(s.sc_theta[j], s.sc_aux[j]);                   // scale of the merged global model
                s.theta[j] = std::fma(alpha, s.inbox[j], keep * s.theta[j]);
            }
            grow(s.sc_theta, s.theta);
            s.snap = s.theta;                                           // theta_{t_last}: the post-merge model
            std::fill(s.acc.begin(), s.acc.end(), R(0));
            std::fill(s.sc_aux.begin(), s.sc_aux.end(), R(0));
            s.phase = ACCUMULATING;
            out.kind = 2;
        }
        out.t = s.t; out.t_last = s.t_last;
        *info = out;
        return 0;
    }

    // GPS block (receive, update, send back) for the Delta that LPS l has in flight.
    int gps_receive(int l) {
        Lps<R> &s = lps[l];
        if (s.phase != SENT) return -2;
        Stopwatch watch(seconds[1], calls[1]);
        gps_updates += 1;
        const bool first = gps_delay.seen == 0, refresh = gps_delay.seen + 1 == gps_delay.d;
        for (int64_t j = 0; j < n; ++j) {
            if (gps_delay.enabled) {
                delayed_update<R>(Theta[j], M[j], gps_buffer[j], s.frozen[j], global, gps_delay.inv_d, first, refresh);
                raise_to(sc_Theta[j], delayed_scales<R>(sc_M[j], sc_gps_buffer[j], M[j], s.sc_aux[j], global,
                                                        gps_delay.inv_d, first, refresh));
                raise_to(sc_Theta[j], std::fabs(Theta[j]));
                continue;
            }
            model_update<R>(Theta[j], M[j], s.frozen[j], global, momentum_bf16);   // ModelUpdate
            raise_to(sc_M[j], s.sc_aux[j]);                             // the scale of G travels with it
            raise_to(sc_M[j], std::fabs(M[j]));
            raise_to(sc_Theta[j], step_scale<R>(sc_M[j], s.sc_aux[j], global));
            raise_to(sc_Theta[j], std::fabs(Theta[j]));
        }
        if (gps_delay.enabled) gps_delay.seen = refresh ? 0 : gps_delay.seen + 1;
        s.inbox = Theta;                                                // send back: this Theta_i, frozen
        s.sc_aux = sc_Theta;
        s.phase = RETURNING;
        return 0;
    }

    // Single tier: the global server applies a worker's delta itself, with its own rule (and its own delayed-momentum
    // cycle if it has one); nothing is sent back -- workers pull the global model.
    int gps_apply_delta(const float *g, float weight) {
        gps_updates += 1;
        const bool first = gps_delay.seen == 0, refresh = gps_delay.seen + 1 == gps_delay.d;
        const R w = R(weight);
        for (int64_t j = 0; j < n; ++j) {
            const R grad = w * R(g[j]);
            R terms;
            if (gps_delay.enabled) {
                delayed_update<R>(Theta[j], M[j], gps_buffer[j], grad, global, gps_delay.inv_d, first, refresh);
                terms = delayed_scales<R>(sc_M[j], sc_gps_buffer[j], M[j], std::fabs(grad), global, gps_delay.inv_d, first, refresh);
            } else {
                model_update<R>(Theta[j], M[j], grad, global, momentum_bf16);
                raise_to(sc_M[j], std::fabs(grad));
                raise_to(sc_M[j], std::fabs(M[j]));
                terms = step_scale<R>(sc_M[j], std::fabs(grad), global);
            }
            raise_to(sc_Theta[j], terms);
            raise_to(sc_Theta[j], std::fabs(Theta[j]));
        }
        if (gps_delay.enabled) { gps_delay.seen = refresh ? 0 : gps_delay.seen + 1; }
        return 0;
    }

    // The message buffer of an LPS as the protocol sees it, by phase: the update accumulated so far
    // (G = theta_{t_last} - theta_t, as a running sum or by subtraction, depending on the form), the frozen G
    // once it has been sent, and the returned global model once the GPS has answered.
    void aux(int l, std::vector<R> &out) const {
        const Lps<R> &s = lps[l];
        out.resize(n);
        if (s.phase == ACCUMULATING) {
            for (int64_t j = 0; j < n; ++j) out[j] = (form == 1) ? s.acc[j] : (s.snap[j] - s.theta[j]);
        } else if (s.phase == SENT) {
            out = s.frozen;
        } else {
            out = s.inbox;
        }
    }
};

struct Handle {
    int precision;
    Oracle<float> *f = nullptr;
    Oracle<double> *d = nullptr;
};

template <class R>
void copy_out(const std::vector<R> &v, double *out) {
    for (size_t j = 0; j < v.size(); ++j) out[j] = (double)v[j];
}

template <class R>
int get_impl(Oracle<R> *o, int what, int l, double *out) {
    const bool per_lps = (what >= 0 && what <= 2) || what == 6 || what == 16 || (what >= 10 && what <= 12) || (what >= 20 && what <= 22);
    if (per_lps && (l < 0 || (size_t)l >= o->lps.size())) return -1;
    switch (what) {
        case 0: copy_out(o->lps[l].theta, out); return 0;
        case 1: copy_out(o->lps[l].m, out); return 0;
        case 2: { std::vector<R> a; o->aux(l, a); copy_out(a, out); return 0; }
        case 6: copy_out(o->lps[l].buffer, out); return 0;
        case 7: copy_out(o->gps_buffer, out); return 0;
        case 16: copy_out(o->lps[l].sc_buffer, out); return 0;
        case 17: copy_out(o->sc_gps_buffer, out); return 0;
        case 3: copy_out(o->Theta, out); return 0;
        case 4: copy_out(o->M, out); return 0;
        case 10: copy_out(o->lps[l].sc_theta, out); return 0;
        case 11: copy_out(o->lps[l].sc_m, out); return 0;
        case 12: copy_out(o->lps[l].sc_aux, out); return 0;
        case 13: copy_out(o->sc_Theta, out); return 0;
        case 14: copy_out(o->sc_M, out); return 0;
        case 20: copy_out(o->lps[l].snap, out); return 0;
        case 21: copy_out(o->lps[l].frozen, out); return 0;
        case 22: copy_out(o->lps[l].inbox, out); return 0;
    }
    return -1;
}

inline float bf16_to_f32(uint16_t bits) { return bf16_value(bits); }

}  // namespace

extern "C" {

void *ho_create(int64_t n, int32_t n_lps, int32_t precision, int32_t form,
                float eta_l, float beta_l, float cg_l, float eta_g, float beta_g, float cg_g,
                float alpha, const int32_t *K, const float *theta0) {
    if (n <= 0 || n_lps <= 0 || (precision != 32 && precision != 64) || (form != 0 && form != 1)) return nullptr;
    Handle *h = new Handle;
    h->precision = precision;
    if (precision == 32)
        h->f = new Oracle<float>(n, n_lps, form, Rule<float>{eta_l, beta_l, cg_l},
                                 Rule<float>{eta_g, beta_g, cg_g}, alpha, K, theta0);
    else
        h->d = new Oracle<double>(n, n_lps, form, Rule<double>{eta_l, beta_l, cg_l},
                                  Rule<double>{eta_g, beta_g, cg_g}, (double)alpha, K, theta0);
    return h;
}

void ho_destroy(void *p) {
    Handle *h = (Handle *)p;
    if (!h) return;
    delete h->f; delete h->d; delete h;
}

#define DISPATCH(call) (h->precision == 32 ? h->f->call : h->d->call)

int ho_arrive_delta_f32(void *p, int32_t l, int32_t worker, const float *g) {
    Handle *h = (Handle *)p;
    return DISPATCH(arrive_delta(l, worker, g));
}

int ho_arrive_delta_bf16(void *p, int32_t l, int32_t worker, const uint16_t *g) {
    Handle *h = (Handle *)p;
    int64_t n = h->precision == 32 ? h->f->n : h->d->n;
    std::vector<float> up(n);
    for (int64_t j = 0; j < n; ++j) up[j] = bf16_to_f32(g[j]);
    return DISPATCH(arrive_delta(l, worker, up.data()));
}

// IEEE binary16 -> binary32, exact (every half value, subnormals included, is a float).
inline float f16_to_f32(uint16_t h) {
    const uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    const uint32_t exp = (h >> 10) & 0x1Fu, frac = h & 0x3FFu;
    uint32_t u;
    if (exp == 0x1Fu) u = sign | 0x7F800000u | (frac << 13);                        // infinity, NaN (payload kept)
    else if (exp != 0) u = sign | ((exp + 112u) << 23) | (frac << 13);              // normal: rebias 15 -> 127
    else if (frac == 0) u = sign;                                                    // zero
    else {                                                                          // subnormal: frac * 2^-24
        float v = (float)frac * 5.9604644775390625e-08f;
        uint32_t b; std::memcpy(&b, &v, sizeof b);
        u = sign | b;
    }
    float f; std::memcpy(&f, &u, sizeof f);
    return f;
}

int ho_arrive_delta_weighted(void *p, int32_t l, int32_t worker, const float *g, float weight) {
    Handle *h = (Handle *)p;
    return DISPATCH(arrive_delta(l, worker, g, weight));
}

// dtype 1: bfloat16 bit patterns, 2: IEEE half bit patterns.
int ho_arrive_delta_16(void *p, int32_t l, int32_t worker, const uint16_t *g, int32_t dtype, float weight) {
    Handle *h = (Handle *)p;
    if (dtype != 1 && dtype != 2) return -1;
    int64_t n = h->precision == 32 ? h->f->n : h->d->n;
    std::vector<float> up(n);
    for (int64_t j = 0; j < n; ++j) up[j] = dtype == 1 ? bf16_to_f32(g[j]) : f16_to_f32(g[j]);
    return DISPATCH(arrive_delta(l, worker, up.data(), weight));
}

int ho_lps_step_average(void *p, int32_t l, int32_t count, void *info) {
    Handle *h = (Handle *)p;
    return DISPATCH(lps_step_average(l, count, (StepInfo *)info));
}

int ho_gps_apply_delta(void *p, const float *g, float weight) {
    Handle *h = (Handle *)p;
    return DISPATCH(gps_apply_delta(g, weight));
}

float ho_f16_to_f32(uint16_t bits) { return f16_to_f32(bits); }

int ho_arrive_global(void *p, int32_t l) { Handle *h = (Handle *)p; return DISPATCH(arrive_global(l)); }

int ho_lps_step(void *p, int32_t l, void *info) {
    Handle *h = (Handle *)p;
    return DISPATCH(lps_step(l, (StepInfo *)info));
}

int ho_gps_receive(void *p, int32_t l) { Handle *h = (Handle *)p; return DISPATCH(gps_receive(l)); }

int ho_set_K(void *p, int32_t l, int32_t K) {
    Handle *h = (Handle *)p;
    if (K < 1) return -1;
    if (h->precision == 32) h->f->lps[l].K = K; else h->d->lps[l].K = K;
    return 0;
}

// Switch a tier to the delayed rule with delay d >= 1 (d = 0: back to plain ModelUpdate).  which: -1 the GPS,
// otherwise the index of an LPS.  Only between cycles.
int ho_set_delay(void *p, int32_t which, int32_t d) {
    Handle *h = (Handle *)p;
    if (d < 0) return -1;
    if (d > 0 && (h->precision == 32 ? h->f->momentum_bf16 : h->d->momentum_bf16)) return -2;
    if (h->precision == 32) {
        auto &dl = which < 0 ? h->f->gps_delay : h->f->lps[which].delay;
        if (dl.seen != 0) return -2;
        if (d == 0) dl = decltype(h->f->gps_delay)(); else dl.set(d);
    } else {
        auto &dl = which < 0 ? h->d->gps_delay : h->d->lps[which].delay;
        if (dl.seen != 0) return -2;
        if (d == 0) dl = decltype(h->d->gps_delay)(); else dl.set(d);
    }
    return 0;
}

// Updates applied since the last momentum refresh (0 .. d-1) of the GPS (which = -1) or an LPS.
int ho_delay_seen(void *p, int32_t which) {
    Handle *h = (Handle *)p;
    if (h->precision == 32) return which < 0 ? h->f->gps_delay.seen : h->f->lps[which].delay.seen;
    return which < 0 ? h->d->gps_delay.seen : h->d->lps[which].delay.seen;
}

int ho_set_rules(void *p, float eta_l, float beta_l, float cg_l, float eta_g, float beta_g, float cg_g, float alpha) {
    Handle *h = (Handle *)p;
    if (h->precision == 32) {
        h->f->local = Rule<float>{eta_l, beta_l, cg_l}; h->f->global = Rule<float>{eta_g, beta_g, cg_g}; h->f->alpha = alpha;
    } else {
        h->d->local = Rule<double>{eta_l, beta_l, cg_l}; h->d->global = Rule<double>{eta_g, beta_g, cg_g}; h->d->alpha = alpha;
    }
    return 0;
}

// what: 0 theta_l, 1 m_l, 2 message buffer of l by phase (accumulated so far / frozen G / returned model),
//       3 Theta, 4 M; 6 gradient buffer of l's delayed momentum, 7 the GPS's; 10..17 the error scales of
//       the same arrays; 20 the snapshot theta_{t_last} of l, 21 the G it last froze, 22 the global model
//       last returned to it (raw state, whatever the phase).
int ho_get(void *p, int32_t what, int32_t l, double *out) {
    Handle *h = (Handle *)p;
    return h->precision == 32 ? get_impl(h->f, what, l, out) : get_impl(h->d, what, l, out);
}

int ho_counters(void *p, int32_t l, int64_t *t, int64_t *t_last, int32_t *phase, int32_t *queued, int64_t *gps_updates) {
    Handle *h = (Handle *)p;
    if (h->precision == 32) {
        auto &s = h->f->lps[l]; *t = s.t; *t_last = s.t_last; *phase = s.phase; *queued = (int32_t)s.queue.size();
        *gps_updates = h->f->gps_updates;
    } else {
        auto &s = h->d->lps[l]; *t = s.t; *t_last = s.t_last; *phase = s.phase; *queued = (int32_t)s.queue.size();
        *gps_updates = h->d->gps_updates;
    }
    return 0;
}

// Stopwatch read-out: seconds[3] and calls[3] for worker updates, GPS updates, merges (see Oracle::Stopwatch).
int ho_stopwatch(void *p, double *seconds, int64_t *calls) {
    Handle *h = (Handle *)p;
    for (int k = 0; k < 3; ++k) {
        seconds[k] = h->precision == 32 ? h->f->seconds[k] : h->d->seconds[k];
        calls[k] = h->precision == 32 ? h->f->calls[k] : h->d->calls[k];
    }
    return 0;
}

int ho_norms(void *p, int32_t l, double *out) {
    Handle *h = (Handle *)p;
    if (h->precision == 32) { out[0] = h->f->lps[l].last_delta_sq; out[1] = h->f->lps[l].last_merge_dist_sq; }
    else { out[0] = h->d->lps[l].last_delta_sq; out[1] = h->d->lps[l].last_merge_dist_sq; }
    return 0;
}

float ho_bf16_to_f32(uint16_t bits) { return bf16_to_f32(bits); }

uint16_t ho_f32_to_bf16(float v) { return f32_to_bf16(v); }

void ho_f32_to_bf16_array(const float *v, int64_t n, uint16_t *out) { for (int64_t j = 0; j < n; ++j) out[j] = f32_to_bf16(v[j]); }

// Keep every server's momentum in bfloat16 from now on (on = 1) or in full precision (0).  Refused (-2) once a momentum
// holds a value that bfloat16 cannot, or while a server runs the delayed rule.
int ho_set_momentum_bf16(void *p, int32_t on) {
    Handle *h = (Handle *)p;
    auto apply = [&](auto *o) -> int {
        if (on) {
            if (o->gps_delay.enabled) return -2;
            for (auto &s : o->lps) if (s.delay.enabled) return -2;
            auto fits = [](const auto &v) {
                for (auto x : v) if ((double)bf16_value(f32_to_bf16((float)x)) != (double)x) return false;
                return true;
            };
            if (!fits(o->M)) return -2;
            for (auto &s : o->lps) if (!fits(s.m)) return -2;
        }
        o->momentum_bf16 = on != 0;
        return 0;
    };
    return h->precision == 32 ? apply(h->f) : apply(h->d);
}

}  // extern "C"
