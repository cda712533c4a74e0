/*
 * gravac_controller.h — C ABI of the host-side adaptive-compression controller (Alg. 1 of the GraVAC
 * paper: the epsilon switch between candidate CF, minimum CF and dense, UpdateStep, CheckGraVAC and the
 * two scaling policies of Sec. IV-B).
 *
 * Pure host code, no GPU call: the controller consumes the per-iteration statistics that
 * gravac_compress / gravac_recompress produce and tells the caller which compression factors to run
 * next and which message to communicate.  One controller object per training job; not thread-safe.
 *
 * Per iteration i = 1, 2, 3, ... the caller
 *   1. calls gravac_controller_candidates  -> theta_min, the candidate CF theta_c and theta_c / theta_min;
 *   2. compresses at theta_min (gravac_compress) and derives the candidate's message from that message
 *      (gravac_recompress at theta_c / theta_min);
 *   3. calls gravac_controller_decide with the two raw gains (both relative to the error-fed gradient)
 *      -> which of the three gradients to communicate (Alg. 1, the three branches on epsilon);
 *   4. communicates, measures the iteration time, and calls gravac_controller_finish_iteration
 *      (UpdateStep, then CheckGraVAC at every multiple of the window).
 *
 * Readings of Alg. 1 where it is silent or at odds with the text (also listed in the design notes):
 *   - EWMA: delta <- alpha * x + (1 - alpha) * delta, started at the first x.  One running value for
 *     theta_min and one for the candidate; the candidate's restarts when the candidate CF changes, and
 *     when theta_min moves up to the candidate it inherits the candidate's running value.
 *   - The candidate CF is min(theta_s * theta_min, theta_max).
 *   - Scale-up of theta_min (gains within omega of each other): theta_min becomes the CF that was just
 *     evaluated, i.e. the candidate of the window that ended (the text's reading; the listing multiplies
 *     by the already re-scaled theta_s, a CF that has no measured gain yet).
 *   - Saturation: when the two largest compression throughputs are within omega of each other, the
 *     ideal CF is the LOWER of the two CFs they belong to (the text's reading; identical to the listing's
 *     lookup in the example the paper gives, 1029.9 at 1280x against 1035.4 at 2000x).
 *   - The returned step theta_ideal / theta_min is not allowed below 1.
 *   - Exponential policy: theta_s <- theta_s^2 (2, 4, 16, 256: powers 2^1, 2^2, 2^4, 2^8);
 *     geometric policy: theta_s <- 2 * theta_s.
 */
#ifndef GRAVAC_CONTROLLER_H
#define GRAVAC_CONTROLLER_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define GRAVAC_POLICY_EXPONENTIAL 0
#define GRAVAC_POLICY_GEOMETRIC   1

/* what to communicate this iteration */
#define GRAVAC_SEND_CANDIDATE 0   /* the message at theta_c; residual follows it */
#define GRAVAC_SEND_MIN       1   /* the message at theta_min */
#define GRAVAC_SEND_DENSE     2   /* the error-fed gradient itself; residual = 0 */

typedef struct gravac_controller gravac_controller;

typedef struct gravac_controller_config {
    double theta_min;              /* >= 1: lower end of the exploration space */
    double theta_max;              /* >= theta_min: upper end */
    double epsilon;                /* in (0, 1]: minimum gain for a CF to be communicated */
    double omega;                  /* >= 0, a fraction (0.01 = 1 %): saturation and scale-up threshold */
    double theta_s;                /* >= 1: initial step (the paper's runs start at 2) */
    double alpha;                  /* in (0, 1]: EWMA factor (the paper: workers / 100) */
    double samples_per_iteration;  /* > 0: workers * per-worker batch size, numerator of T_sys */
    int64_t window;                /* >= 1: iterations per candidate CF */
    int32_t policy;                /* GRAVAC_POLICY_* */
    int32_t reserved;              /* must be 0 */
} gravac_controller_config;

/* Creates a controller.  Returns GRAVAC_OK or GRAVAC_ERR_INVALID_ARG; *out is NULL on error.
 * The caller owns the object and releases it with gravac_controller_destroy (NULL is allowed). */
int gravac_controller_create(const gravac_controller_config* config, gravac_controller** out);
void gravac_controller_destroy(gravac_controller* c);

/* The CFs of the coming iteration: theta_min, the candidate theta_c = min(theta_s * theta_min,
 * theta_max), and cf_rel = theta_c / theta_min (the second-level factor).  Any output may be NULL. */
int gravac_controller_candidates(const gravac_controller* c, double* theta_min, double* theta_c, double* cf_rel);

/* Alg. 1, gain steps and the epsilon branches.  gain_min and gain_c are this iteration's raw
 * ||g_min||^2/||g_o||^2 and ||g_c||^2/||g_o||^2 (finite, >= 0).  Outputs: choice = GRAVAC_SEND_*,
 * delta_min / delta_c = the smoothed gains (may be NULL).  Must be followed by
 * gravac_controller_finish_iteration before the next decide. */
int gravac_controller_decide(gravac_controller* c, double gain_min, double gain_c,
                             int32_t* choice, double* delta_min, double* delta_c);

/* Alg. 1, UpdateStep for the branch taken (t_iter > 0 seconds: T_sys = samples_per_iteration / t_iter,
 * T_compress[theta] = T_sys * delta) and CheckGraVAC when the iteration number is a multiple of the
 * window.  theta_s_out (may be NULL) receives the step for the next iteration. */
int gravac_controller_finish_iteration(gravac_controller* c, double t_iter, double* theta_s_out);

/* T_compress[cf] as last recorded; returns GRAVAC_ERR_INVALID_ARG if that CF has no entry. */
int gravac_controller_throughput(const gravac_controller* c, double cf, double* t_compress);

/* Number of iterations finished so far. */
int64_t gravac_controller_iteration(const gravac_controller* c);

#ifdef __cplusplus
}
#endif
#endif
