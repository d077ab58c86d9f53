/* C ABI of the Resource-Aware Dispatcher's integer program (host code only, no GPU).
 *
 * The program (Section "Resource-Aware Dispatcher", "Solution for Gamma^D": objective (OBJ),
 * constraints (C0)-(C4)): requests r, Primary-replica types i (at most 4: <EDC>, <DC>, <ED>,
 * <D>), parallel degrees k (at most 4, the set {1,2,4,8}); binary x[r][i][k] dispatches r
 * now on k idle replicas of type i.
 *
 *   maximise   sum (W[r] - Q[r][i]) x[r][i][k]
 *   subject to x <= feas (= E[r][k] * F[r][i][k], computed by the caller)       (C0)
 *              at most one (i,k) per request                                    (C1)
 *              sum over r,k of k * x[r][i][k] <= B[i] for every type i          (C2)
 *              D[r] = 1 only if r is dispatched and tau + t[r][i][k] <= d[r]    (C3a, C3b)
 *
 * D does not occur in the objective; it is reported as the largest value the constraints
 * allow.  The objective does not depend on k, so of several feasible degrees on one type
 * the smallest is taken (it leaves the most replicas to others).
 *
 * All arrays are host memory, row-major, owned by the caller: t, feas: [R][I][K];
 * W, deadline, length: [R]; Q: [R][I]; B, beta: [I]; degrees: [K], positive, ascending.
 * Return value: TDS_OK, TDS_LIMIT (node limit reached: the best assignment found so far is
 * returned, *upper_bound says how far it can be from the optimum) or TDS_EINVAL (null
 * pointer, R < 0, I or K outside 1..4, non-positive or unsorted degrees, negative B, a
 * non-finite number): then no output is written.
 */
#ifndef TDS_DISPATCH_H
#define TDS_DISPATCH_H

#ifdef __cplusplus
extern "C" {
#endif

enum { TDS_OK = 0, TDS_LIMIT = 1, TDS_EINVAL = -1 };

/* SLO-aware reward (Appendix "Dispatch Plan", the W_r equation): with T_hat = min over
 * feasible (i,k) of tau + t[r][i][k] and scale = max(1, T_hat / d[r]):
 * W[r] = c_on if T_hat <= d[r], else c_late * max(1, scale - alpha + 1); 0 when nothing is
 * feasible.  The paper's constants: c_on 1000, c_late 200, alpha 5. */
int tds_reward_weights(int R, int I, int K, const double* t, const unsigned char* feas,
                       const double* deadline, double tau, double c_on, double c_late,
                       double alpha, double* W);

/* Communication penalty (the Q_{r,i} equation): Q[r][i] = beta[i] * length[r]; the paper's
 * beta: 0, 1e-6, 5e-6, 6e-6 for <EDC>, <DC>, <ED>, <D>. */
int tds_comm_penalty(int R, int I, const double* length, const double* beta, double* Q);

/* Solves the program by branch and bound (depth first, Lagrangian bound with the replica
 * counts rounded to usable multiples).  choice_type[r], choice_degree[r]: the chosen type
 * index and degree (the value k, not its index), or -1, -1 when r stays undispatched;
 * D: [R]; *objective: value of (OBJ); *upper_bound: a proven upper bound on the optimum
 * (== *objective up to rounding when TDS_OK); *nodes: search nodes visited.  node_limit
 * <= 0 means no limit.  gap_abs >= 0: the search stops as soon as upper bound - objective
 * <= gap_abs (0 = prove optimality). */
int tds_dispatch_solve(int R, int I, int K, const int* degrees, const double* W,
                       const double* Q, const unsigned char* feas, const int* B,
                       const double* t, const double* deadline, double tau,
                       long long node_limit, double gap_abs, int* choice_type,
                       int* choice_degree, unsigned char* D, double* objective,
                       double* upper_bound, long long* nodes);

#ifdef __cplusplus
}
#endif
#endif
