/*
 * ukv_sched.h -- C ABI of the request scheduler that feeds the unified-KV path: SeaLLM's
 * doubling-budget (DB) algorithm (arXiv 2504.15720, section 4.2 "Latency-Optimized Scheduling",
 * Equation 6, and the DB scheduling algorithm of the appendix).  Host code only.
 *
 * Every request r of service s carries a budget Q_r, initially Q = L_s + Var_s (mean and standard
 * deviation of the execution time of that service's requests), and a priority O_r = Q_r * L_s; the
 * smallest O_r is served first.  The budget decreases with the time r executes; when it is used up
 * and r is not finished it becomes 2Q, then 4Q, ... and the priority is reset from it.  Requests wait
 * in two priority queues (not yet prefilled / decoding); a batch holds requests of ONE service in
 * ONE phase, taken in priority order from the queue of the chosen request while EnoughResource()
 * holds.  A service whose queued requests have not been served for longer than its starvation
 * threshold is served first.
 *
 * Readings where the paper is silent: an iteration's execution time is charged in full to every
 * request of its batch; EnoughResource() = fewer than max_batch requests and the pages the batch's
 * next iteration needs (the whole prompt for a prefill, the growth by one token for a decode) fit
 * in free_pages, the number of free pages the caller reports (normally ukv_pool_info().free_pages
 * of the pool the requests live in); a candidate that does not fit ends the batch; if the chosen
 * request itself does not fit, the next request in the same order that fits is chosen; ties go to
 * the earlier arrival, then the smaller id; a service's starvation clock starts with its first
 * queued request and restarts when one of its batches completes.
 *
 * The scheduler allocates no pages and touches no device memory: the caller executes the batch
 * (ukv_scatter + ukv_prefill_attention, or ukv_decode_step) and reports back.  Not thread-safe.
 * Errors and ukv_last_error() as in ukv.h.
 */
#ifndef UKV_SCHED_H
#define UKV_SCHED_H

#include "ukv.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ukv_sched ukv_sched_t; /* opaque host object */

typedef struct {
    double mean_time;            /* L_s: profiled execution time of a request of the service */
    double std_time;             /* Var_s: its standard deviation */
    double starvation_threshold; /* same unit as the clock the caller passes as `now` */
} ukv_sched_service_t;

#define UKV_SCHED_WAIT 0     /* wait_queue: not yet prefilled */
#define UKV_SCHED_DECODING 1 /* decoding_queue */

typedef struct {
    uint32_t service, queue, prompt_len, ctx_len, doublings;
    double arrival, budget, priority;
} ukv_sched_request_t;

/* services: HOST [n], n = the pool's number of services (token sizes and the page size are taken
 * from the pool at this call; the pool is not referenced afterwards).  max_batch >= 1. */
int ukv_sched_create(const ukv_pool_t *pool, const ukv_sched_service_t *services, uint32_t n_services,
                     uint32_t max_batch, ukv_sched_t **out);
int ukv_sched_destroy(ukv_sched_t *sched);

/* A new request arrives: InitBudget, InitPriority, wait_queue.AddRequest.  id must be unused,
 * prompt_len >= 1. */
int ukv_sched_add_request(ukv_sched_t *sched, uint64_t id, uint32_t service, uint32_t prompt_len, double now);

/* "Schedule requests": the next batch to execute.  ids_out HOST [cap] receives *n_out ids in
 * priority order (cap >= max_batch); *service_out and *queue_out name the batch's service and
 * phase.  *n_out == 0: nothing queued, or nothing that fits free_pages. */
int ukv_sched_next_batch(ukv_sched_t *sched, double now, uint64_t free_pages, uint64_t *ids_out, uint32_t cap,
                         uint32_t *n_out, uint32_t *service_out, uint32_t *queue_out);

/* The batch (as returned by the last ukv_sched_next_batch) has executed for `elapsed`: prefilled
 * requests move to the decoding queue with ctx_len = prompt_len, decoded ones gain a token;
 * finished[i] != 0 removes request ids[i]; the others get UpdateBudget / UpdatePriority. */
int ukv_sched_complete(ukv_sched_t *sched, const uint64_t *ids, const uint8_t *finished, uint32_t n, double elapsed,
                       double now);

/* Pages the next iteration of request id would take from the free list. */
int ukv_sched_pages_needed(const ukv_sched_t *sched, uint64_t id, uint64_t *pages_out);
int ukv_sched_request_info(const ukv_sched_t *sched, uint64_t id, ukv_sched_request_t *out);
uint32_t ukv_sched_pending(const ukv_sched_t *sched); /* requests in the two queues; 0 on a null handle */

#ifdef __cplusplus
}
#endif
#endif /* UKV_SCHED_H */
