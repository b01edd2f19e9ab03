/*
 * cdsgd_cost_model.h -- the paper's per-iteration time model (Sec. 2.1-2.3, Sec. 3.3)
 * as a host-side calculator: feed it the measured compression time delta and it
 * returns the iteration times of S-SGD, the local-update mechanism, BIT-SGD and
 * CD-SGD and what CD-SGD saves against the latter two.
 *
 * Symbols (Table 1): tau = computation time per iteration, phi = uncompressed
 * communication time, psi = compressed communication time, delta = extra time
 * brought by compression, k = correction period.  All times in the same unit,
 * finite and >= 0.  Host memory only; nothing here touches the GPU.
 *
 *   T_ssgd  = tau + phi                                             (eq. 2)
 *   T_loc   = tau if tau > phi, phi if tau < phi                    (eq. 4; a tie gives tau = phi)
 *   T_bit   = tau + delta + psi                                     (eq. 5)
 *   phi_cd  = delta + psi if i mod k != 0, phi if i mod k == 0      (eq. 6)
 *   T_cd    = tau if tau > phi_cd, else phi_cd                      (eq. 7; a tie gives the same value)
 *   save_vs_bit, save_vs_loc: the case tables of eq. 8 and eq. 9
 *
 * The case table of eq. 9 tacitly assumes delta + psi <= phi (compression pays
 * off on the wire); outside that regime save_vs_loc follows the table as printed
 * and differs from T_loc - T_cd, and `eq9_assumption_holds` is 0.
 */
#ifndef CDSGD_COST_MODEL_H
#define CDSGD_COST_MODEL_H

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    double tau, phi, psi, delta;
    int k;
} cdsgd_cost_params;

typedef struct {
    double t_ssgd, t_loc, t_bit;  /* eq. 2, 4, 5 */
    double phi_cd, t_cd;          /* eq. 6, 7 */
    double save_vs_bit;           /* eq. 8 */
    double save_vs_loc;           /* eq. 9 */
    int case_bit;                 /* which case of eq. 8 applied (1..3) */
    int case_loc;                 /* which case of eq. 9 applied (1..4) */
    int eq9_assumption_holds;     /* delta + psi <= phi */
} cdsgd_cost;

/* Iteration i (>= 0) of the model.  Returns 0, or 3 (CDSGD_ERR_PARAM) for a NULL
 * pointer, k < 1, i < 0 or a time that is negative or not finite. */
int cdsgd_cost_iteration(const cdsgd_cost_params *p, long i, cdsgd_cost *out);

/* Means over one period of k iterations (i = 0 .. k-1) of every field of
 * cdsgd_cost that is a time; the case fields are 0.  When communication
 * dominates (tau < delta + psi and tau < phi) t_cd is ((k-1)(delta+psi)+phi)/k
 * (Sec. 3.3). */
int cdsgd_cost_period_mean(const cdsgd_cost_params *p, cdsgd_cost *out);

#ifdef __cplusplus
}
#endif
#endif
