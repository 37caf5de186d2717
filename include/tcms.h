/*
 * tcms.h - C ABI of the scheduling front-end that decides in which order requests
 * enter the vision encoder (host code only; part of libtcmv.so).
 *
 * It follows the components of the paper's Section 3 (Fig. 5):
 *   Impact Estimator   (Sec. 3.3)  tcms_fit_linear, tcms_fit_quantile, tcms_pinball_loss
 *   Request Classifier (Sec. 3.4)  tcms_classify_naive, tcms_cluster_fit, tcms_cluster_assign
 *   Queue Manager      (Sec. 3.5)  tcms_queues_*
 *   Priority Regulator (Sec. 3.6)  tcms_priority, tcms_score, tcms_regulator_default
 *   and a trace-driven model of one non-preemptive server, tcms_simulate, to compare the
 *   policies the paper compares in Sec. 3.4 / 3.6 (FCFS, static priority, regulated).
 *
 * All pointers are HOST pointers owned by the caller unless stated otherwise; arrays
 * are contiguous.  Functions return TCMS_OK (0) or a negative TCMS_E_* code and write
 * nothing to their outputs on error.  Nothing here touches the GPU.  Functions are
 * re-entrant; a tcms_queues object must not be used from two threads at once.
 *
 * Classes (Sec. 3.1, the trucks / cars / motorcycles abstraction): the smaller the code,
 * the lighter the request.
 */
#ifndef TCMS_H
#define TCMS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { TCMS_MOTORCYCLE = 0, TCMS_CAR = 1, TCMS_TRUCK = 2 };
enum { TCMS_FCFS = 0, TCMS_STATIC = 1, TCMS_REGULATED = 2 };
enum { TCMS_OK = 0, TCMS_E_INVALID_ARG = -1, TCMS_E_EMPTY = -2, TCMS_E_DEGENERATE = -3 };

/* ---- Impact Estimator (Sec. 3.3) -------------------------------------------------------
 * The paper predicts a request's cost from its size with a linear regression for text and
 * with a quantile regression at the 90th percentile for image and video requests, so that
 * heavy requests are not underestimated. */

/* Ordinary least squares y ~ intercept + slope*x over n >= 1 points.  If all x are equal
 * the slope is 0 and the intercept the mean of y. */
int tcms_fit_linear(const double* x, const double* y, int64_t n, double* slope, double* intercept);

/* Sum over the points of rho_q(y - intercept - slope*x), rho_q(r) = q*r (r >= 0), (q-1)*r (r < 0). */
double tcms_pinball_loss(const double* x, const double* y, int64_t n, double q, double slope, double intercept);

/* Quantile regression at level 0 < q < 1: a line minimising tcms_pinball_loss, found exactly
 * (the optimum of the underlying linear program is a line through two data points; for every
 * point the best line through it is a weighted quantile of the slopes to the other points).
 * O(n^2 log n) time, O(n) memory.  *loss (may be NULL) receives the minimum.  If all x are
 * equal the slope is 0 and the intercept a q-quantile of y.  The minimising line need not be
 * unique; the minimum is. */
int tcms_fit_quantile(const double* x, const double* y, int64_t n, double q, double* slope, double* intercept,
                      double* loss);

/* The same two fits with a second regressor, y ~ coef[0] + coef[1]*x1 + coef[2]*x2.  It is meant for
 * x1 = tokens of a request and x2 = sum of its squared attention-segment lengths: the attention
 * work of the vision encoder grows with x2, everything else with x1, so this is the smallest model
 * that follows both short images and long videos.  coef: 3 doubles, written by the call.
 * tcms_fit_linear2: a constant regressor gets coefficient 0; proportional regressors share the slope
 * (minimum-norm solution of the centred, scaled problem).  tcms_fit_quantile2: exact (the optimum is
 * a plane through three data points; for every pair of points the best plane through both is a
 * weighted quantile), O(n^3 log n) time, n <= 4096; the minimum is unique, the plane need not be. */
int tcms_fit_linear2(const double* x1, const double* x2, const double* y, int64_t n, double* coef);
double tcms_pinball_loss2(const double* x1, const double* x2, const double* y, int64_t n, double q,
                          const double* coef);
int tcms_fit_quantile2(const double* x1, const double* x2, const double* y, int64_t n, double q, double* coef,
                       double* loss);

/* ---- Request Classifier (Sec. 3.4) ----------------------------------------------------- */

/* The paper's "naive" rule: modality 0 text -> motorcycle, 1 image -> car, 2 video -> truck;
 * TCMS_E_INVALID_ARG otherwise. */
int tcms_classify_naive(int modality);

/* The paper's "smart" classifier is a clustering model with three clusters over the two
 * outputs of the Impact Estimator.  Here: k-means (Lloyd's iterations) on
 * (log(1+time), log(1+tokens)), each standardised to zero mean and unit variance; initial
 * centroids = the requests at the 1/6, 3/6 and 5/6 quantiles of the first feature; ties go to
 * the lower cluster; clusters are numbered by increasing first coordinate of their centroid,
 * so cluster 0 = motorcycles, 1 = cars, 2 = trucks. */
typedef struct {
  double mean[2], scale[2]; /* standardisation of the two log features */
  double centroid[3][2];    /* in standardised log space, ordered by centroid[.][0] */
} tcms_cluster_model;

/* features: [n][2] = (time, tokens), all >= 0, n >= 3.  max_iter >= 1 bounds the iterations. */
int tcms_cluster_fit(const double* features, int64_t n, int max_iter, tcms_cluster_model* out);
/* Class (0..2) of one request; negative code on invalid input. */
int tcms_cluster_assign(const tcms_cluster_model* m, double time, double tokens);

/* ---- Priority Regulator (Sec. 3.6) ------------------------------------------------------
 * Priority_c = static_priority[c] + (1 - exp(-k[c] * wait^p[c])),  Score_c = -log(Priority_c);
 * the request with the lowest score is served next.  Score is +infinity when Priority is 0. */
typedef struct { double static_priority[3], k[3], p[3]; } tcms_regulator;

/* The constants of the paper's evaluation (Sec. 4.1, "Configuration"). */
void tcms_regulator_default(tcms_regulator* r);
double tcms_priority(const tcms_regulator* r, int cls, double wait);
double tcms_score(const tcms_regulator* r, int cls, double wait);

/* ---- Queue Manager (Sec. 3.5) -----------------------------------------------------------
 * Three FCFS queues, one per class.  pop returns the request to serve next at time `now`:
 *   TCMS_FCFS       earliest arrival over all queues,
 *   TCMS_STATIC     head of the lightest non-empty class,
 *   TCMS_REGULATED  head with the lowest score at `now` (earliest arrival on ties).
 * Inside a class the head is always the best candidate because the age term grows with the
 * wait.  Requests must be pushed in non-decreasing arrival order per class. */
typedef struct tcms_queues tcms_queues; /* opaque; freed by tcms_queues_destroy */

tcms_queues* tcms_queues_create(const tcms_regulator* r, int policy); /* NULL on invalid arguments */
void tcms_queues_destroy(tcms_queues* q);
int tcms_queues_push(tcms_queues* q, int64_t id, int cls, double arrival);
/* TCMS_E_EMPTY when nothing waits. */
int tcms_queues_pop(tcms_queues* q, double now, int64_t* id, int* cls, double* arrival);
/* Load metrics the paper's Queue Manager tracks: length and mean waiting time (at `now`) per class. */
int tcms_queues_stats(const tcms_queues* q, double now, int64_t length[3], double mean_wait[3]);

/* ---- one non-preemptive server over a trace ----------------------------------------------
 * arrival (non-decreasing), service (>= 0) and cls (0..2) describe n requests; start[i]
 * receives the time request i enters service under `policy`. */
int tcms_simulate(const tcms_regulator* r, int policy, int64_t n, const double* arrival, const double* service,
                  const int32_t* cls, double* start);

#ifdef __cplusplus
}
#endif
#endif /* TCMS_H */
