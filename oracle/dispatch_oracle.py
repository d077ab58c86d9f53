"""Reference for the Resource-Aware Dispatcher's integer program (TEST INFRASTRUCTURE).

Plain, slow and exhaustive: the reward weights and communication penalties written out from
their defining equations, and the dispatch problem solved by enumerating every assignment.
Only tests (and a benchmark's CPU-baseline leg) may import this module; the product solver
shares no code with it.

What is computed (Section "Resource-Aware Dispatcher", "Solution for Gamma^D": sets, (OBJ),
(C0)-(C4); Appendix "Dispatch Plan": the W_r and Q_{r,i} equations and the constant values):

  maximise   sum_{r,i,k} (W_r - Q_{r,i}) x_{r,i,k}
  subject to x_{r,i,k} <= E_{r,k} F_{r,i,k}                     (C0)  [feas = E*F, given]
             sum_{i,k} x_{r,i,k} <= 1              for every r   (C1)
             sum_{r,k} k x_{r,i,k} <= B_i          for every i   (C2)
             tau + sum t x <= d_r + M (1 - D_r),  D_r <= sum x   (C3a, C3b)
             x, D binary                                          (C4)

D_r does not occur in the objective, so it never changes the optimum; it is reported as the
largest value (C3a)/(C3b) allow: 1 iff r is dispatched and tau + t <= d_r.
"""
import itertools

import numpy as np

C_ON, C_LATE, ALPHA = 1000.0, 200.0, 5.0                 # Appendix "Dispatch Plan", constant values
BETA = (0.0, 1e-6, 5e-6, 6e-6)                           # types <EDC>, <DC>, <ED>, <D>
DEGREES = (1, 2, 4, 8)


def reward_weights(t, feas, deadline, tau, c_on=C_ON, c_late=C_LATE, alpha=ALPHA):
    """W_r of the W_r equation.  t, feas: [R][I][K]; deadline: [R].

    T_hat_r = min over feasible (i,k) of tau + t[r,i,k]; scale_r = max(1, T_hat_r / d_r);
    W_r = c_on if T_hat_r <= d_r else c_late * max(1, scale_r - alpha + 1).
    A request with no feasible option gets W_r = 0 (it cannot be dispatched at all).
    """
    t = np.asarray(t, np.float64)
    feas = np.asarray(feas).astype(bool)
    R = t.shape[0]
    W = np.zeros(R)
    for r in range(R):
        if not feas[r].any():
            continue
        t_hat = tau + t[r][feas[r]].min()
        if t_hat <= deadline[r]:
            W[r] = c_on
        else:
            scale = max(1.0, t_hat / deadline[r])
            W[r] = c_late * max(1.0, scale - alpha + 1.0)
    return W


def comm_penalty(length, beta=BETA):
    """Q_{r,i} = beta_i * l_r (the Q_{r,i} equation)."""
    return np.outer(np.asarray(length, np.float64), np.asarray(beta, np.float64))


def objective(choice, W, Q):
    """Value of (OBJ) for choice[r] = (i, k) or None."""
    return sum(W[r] - Q[r][c[0]] for r, c in enumerate(choice) if c is not None)


def on_time(choice, t, deadline, tau, degrees=DEGREES):
    """D_r: 1 iff dispatched and tau + t_{r,i,k} <= d_r."""
    out = []
    for r, c in enumerate(choice):
        out.append(int(c is not None and tau + t[r][c[0]][degrees.index(c[1])] <= deadline[r]))
    return out


def solve_bruteforce(W, Q, feas, B, degrees=DEGREES):
    """Every assignment of every request to 'none' or one feasible (type, degree); keeps the
    feasible one (C2) of largest (OBJ).  Returns (best objective, one maximiser)."""
    feas = np.asarray(feas).astype(bool)
    R, I, K = feas.shape
    options = []
    for r in range(R):
        opts = [None] + [(i, degrees[k]) for i in range(I) for k in range(K) if feas[r, i, k]]
        options.append(opts)
    best, arg = -1.0, None
    for choice in itertools.product(*options):
        used = [0] * I
        for c in choice:
            if c is not None:
                used[c[0]] += c[1]
        if any(used[i] > B[i] for i in range(I)):
            continue
        v = objective(choice, W, Q)
        if v > best:
            best, arg = v, choice
    return best, list(arg)
