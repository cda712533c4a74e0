"""CPU oracle of the adaptive-compression controller (Alg. 1 of the GraVAC paper).

TEST INFRASTRUCTURE ONLY: imported by the tests, never by the product package, and it imports nothing
from the product package.  Plain Python in the listing's order and notation: one call of ``iteration``
is one pass through the body of the training loop of Alg. 1 (gain steps, the epsilon branches,
UpdateStep, CheckGraVAC); gradients, compression and communication are replaced by two callables that
give the raw gain of a CF and the iteration time of the branch taken.

Readings where the listing is silent or differs from the text (Sec. III-C, Sec. IV-B):
  * EWMA(x): delta = alpha * x + (1 - alpha) * delta, the first value is x itself.  delta_c restarts when
    the candidate CF changes; when theta_min moves up to the candidate it takes delta_c's history along.
  * candidate CF = min(theta_s * theta_min, theta_max).
  * scale-up of theta_min: to the candidate CF of the window that just ended (text of Sec. III-C).
  * saturation: theta_ideal is the lower of the two CFs that hold the two largest compression
    throughputs (text of Sec. III-C; same as the listing's lookup in the example of Sec. IV-B).
  * theta_s never drops below 1.
  * ScalingPolicy: exponential squares theta_s (2, 4, 16, 256), geometric doubles it (Sec. IV-B).
"""
from __future__ import annotations

SEND_CANDIDATE, SEND_MIN, SEND_DENSE = 0, 1, 2


class State:
    def __init__(self, theta_min, theta_max, epsilon, omega, window, policy, theta_s=2.0, alpha=0.32, N_b=1.0):
        self.theta_min = float(theta_min)
        self.theta_max = float(theta_max)
        self.epsilon = float(epsilon)
        self.omega = float(omega)
        self.window = int(window)
        self.policy = policy                      # "exponential" | "geometric"
        self.theta_s = float(theta_s)
        self.alpha = float(alpha)
        self.N_b = float(N_b)                     # workers * per-worker batch size
        self.i = 0
        self.delta_min = None                     # EWMA values (None = no sample yet)
        self.delta_c = None
        self.T_compress = {}                      # CF -> compression throughput


def _ewma(old, x, alpha):
    return x if old is None else alpha * x + (1.0 - alpha) * old


def _scaling_policy(policy, theta_s):
    if policy == "exponential":
        return theta_s * theta_s
    if policy == "geometric":
        return 2.0 * theta_s
    raise ValueError(policy)


def candidate(st: State) -> float:
    return min(st.theta_s * st.theta_min, st.theta_max)


def _check_gravac(st: State):
    evaluated = candidate(st)
    st.theta_s = _scaling_policy(st.policy, st.theta_s)
    # scale-up of the minimum CF
    if st.delta_min > 0.0 and st.omega >= abs(st.delta_min - st.delta_c) / st.delta_min and evaluated > st.theta_min:
        st.theta_min = evaluated
        st.delta_min = st.delta_c
    # saturation of the compression throughput
    if len(st.T_compress) >= 2:
        best = second = None                      # (throughput, CF); equal throughputs: the lower CF ranks higher
        for cf, t in st.T_compress.items():
            entry = (t, -cf)
            if best is None or entry > best:
                best, second = entry, best
            elif second is None or entry > second:
                second = entry
        ct_1, ct_2 = best[0], second[0]
        if ct_2 > 0.0 and abs((ct_1 - ct_2) / ct_2) <= st.omega:
            theta_ideal = min(-best[1], -second[1])
            st.theta_s = max(1.0, theta_ideal / st.theta_min)
    if candidate(st) != evaluated:
        st.delta_c = None


def iteration(st: State, gain_of, time_of) -> dict:
    """One training iteration of Alg. 1.

    ``gain_of(cf)`` -> raw ||g_cf||^2 / ||g_o||^2 of this iteration; ``time_of(choice, cf)`` -> t_iter of
    the branch taken (cf = 1 for dense).  Returns what happened in a dict.
    """
    st.i += 1
    theta_min = st.theta_min
    theta_c = candidate(st)
    st.delta_min = _ewma(st.delta_min, gain_of(theta_min), st.alpha)
    st.delta_c = _ewma(st.delta_c, gain_of(theta_c), st.alpha)
    delta_min, delta_c = st.delta_min, st.delta_c
    if delta_c >= st.epsilon:
        choice, theta, delta = SEND_CANDIDATE, theta_c, delta_c
    elif delta_min >= st.epsilon:
        choice, theta, delta = SEND_MIN, theta_min, delta_min
    else:
        choice, theta, delta = SEND_DENSE, 1.0, 1.0
    t_iter = time_of(choice, theta)
    # UpdateStep
    T_sys = st.N_b / t_iter
    st.T_compress[theta] = T_sys * delta
    # CheckGraVAC
    if st.i % st.window == 0:
        _check_gravac(st)
    return {"i": st.i, "theta_min": theta_min, "theta_c": theta_c, "choice": choice, "cf_used": theta,
            "delta_min": delta_min, "delta_c": delta_c, "t_iter": t_iter, "theta_s_next": st.theta_s,
            "theta_min_next": st.theta_min}
