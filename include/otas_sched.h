/* Host side of OTAS: the batch queue with adaptive batching (Sec. III-C, Alg. 1) and online token
 * adaptation (Sec. III-D: the dynamic program of Alg. 2, its rate-driven fallback Alg. 3, and the
 * profile-based estimates of a batch's processing time and utility).  It produces the per-batch gamma
 * (P prompt tokens when gamma > 0, r merged tokens per layer when gamma < 0) that otas_encoder_forward
 * takes as input.
 *
 * Everything here runs on the host and touches no device: all pointers are HOST pointers, all times are
 * seconds as double on one clock chosen by the caller.  A scheduler object is not thread safe.
 * Functions return a status code of otas.h (OTAS_OK = 0); on any error the queue is left as it was.
 */
#ifndef OTAS_SCHED_H_
#define OTAS_SCHED_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct otas_sched otas_sched;

/* Thresholds of Alg. 1 (delta, epsilon, eta, mu), of Alg. 2 (beta) and of Alg. 3 (kappa).  The paper's
 * experiment uses delta = 0.5 s, epsilon = 64, eta = 0.5 s, mu = 0.8, beta = 5, kappa = 0.8 (Sec. V). */
typedef struct {
  double delta;     /* longest wait of a batch's first request before the batch stops accepting  */
  double eta;       /* largest |d_b - d_r| for r to join b                                        */
  double mu;        /* largest |u_b - u_r| for r to join b                                        */
  double kappa;     /* Alg. 3: mean utility above which a batch gets the largest gamma            */
  int32_t epsilon;  /* largest batch size, >= 1                                                   */
  int32_t beta;     /* Alg. 2: queues of at most beta batches take Alg. 3                         */
} otas_sched_params;

#define OTAS_GAMMA_SKIP (-1)      /* Alg. 2 decided not to execute the batch                     */
#define OTAS_GAMMA_UNDECIDED (-2) /* no allocation pass has seen the batch yet                   */

/* Creates a scheduler.  gammas[n_gamma]: the selection list L^(gamma), any order, distinct values.
 * latency[n_tasks * n_gamma], accuracy[n_tasks * n_gamma]: row-major [task][index into gammas], the
 * profiled per-sample latency in seconds (> 0) and accuracy of each task at each gamma (Sec. III-D,
 * last paragraphs).  rate_max[n_rate] ascending and rate_gamma[n_rate] (indices into gammas): the
 * projection f of Alg. 3 / Table I: a request rate q takes the first row with q <= rate_max, a rate
 * above every row takes the smallest gamma of the list; n_rate may be 0.  All arrays are copied.
 * OTAS_EINVAL on NULL pointers, non-positive counts, indices out of range, unsorted rate_max. */
int otas_sched_create(const otas_sched_params* params, int32_t n_gamma, const int32_t* gammas, int32_t n_tasks,
                      const double* latency, const double* accuracy, int32_t n_rate, const double* rate_max,
                      const int32_t* rate_gamma, otas_sched** out);
void otas_sched_destroy(otas_sched* s);

/* The projection f of Alg. 3 built from a latency profile (Sec. III-D; Table I is the paper's instance for
 * its own machine): walking the selection list from the largest gamma down, a gamma serves every request
 * rate up to its own throughput 1 / (mean over tasks of the per-sample latency); a gamma whose throughput
 * does not exceed the previous row's gets no row; the smallest gamma gets none either (rates above the
 * table take it).  latency as in otas_sched_create.  Outputs: rate_max[*n_rate] ascending and
 * rate_gamma[*n_rate] (indices into gammas), arrays of at least n_gamma - 1 entries, ready for
 * otas_sched_create.  Pure host function. */
int otas_sched_rate_table(int32_t n_gamma, const int32_t* gammas, int32_t n_tasks, const double* latency,
                          double* rate_max, int32_t* rate_gamma, int32_t* n_rate);

/* Alg. 1: puts request `id` (arrival time s_r, latency requirement l_r, utility u_r, task) into the newest
 * acceptable batch of the queue, walking from its last batch towards its first, or opens a new batch at
 * the end.  *batch (may be NULL) receives the queue position of the batch that took it. */
int otas_sched_add_query(otas_sched* s, int64_t id, double s_r, double l_r, double u_r, int32_t task,
                         int32_t* batch);

/* Alg. 2 at clock time T with estimated arriving rate q (requests / s): sorts the queue by batch deadline
 * (stable) and gives every batch an index into gammas or OTAS_GAMMA_SKIP; with at most beta batches, or
 * with initial_stage != 0, Alg. 3 decides instead.  *planned_utility (may be NULL) receives the dynamic
 * program's best accumulated utility, or NaN when Alg. 3 decided.  An empty queue is not an error. */
int otas_sched_allocate(otas_sched* s, double T, double q, int32_t initial_stage, double* planned_utility);

/* Queue inspection.  Positions are 0-based in queue order.  Any output pointer may be NULL. */
int32_t otas_sched_num_batches(const otas_sched* s);
int otas_sched_batch_info(const otas_sched* s, int32_t b, int32_t* size, double* s_b, double* d_b, double* u_b,
                          int32_t* gamma_index);
/* Copies up to cap request ids / tasks of batch b in arrival order; *n (may be NULL) = batch size. */
int otas_sched_batch_queries(const otas_sched* s, int32_t b, int64_t* ids, int32_t* tasks, int32_t cap,
                             int32_t* n);
/* Profile(B_b, gammas[gamma_index]): estimated processing time (sum over tasks, ascending, of the task's
 * request count times its per-sample latency) and utility (sum over requests in arrival order of
 * u_r times the accuracy of r's task). */
int otas_sched_estimate(const otas_sched* s, int32_t b, int32_t gamma_index, double* t_hat, double* U_hat);
/* Removes batch b from the queue (it was executed, or given up). */
int otas_sched_remove(otas_sched* s, int32_t b);

#ifdef __cplusplus
}
#endif
#endif /* OTAS_SCHED_H_ */
