/*
 * TD-Pipe control decisions as a host library (no GPU, no dependencies): C ABI of libtdp_sched.so.
 *
 * The paper's engine (Sec. 3.2.1) decides, from memory capacity, request status and profiling
 * results, which batch each worker runs in which phase.  These are the three decisions it names,
 * plus a simulated n-stage pipeline that is driven by them and timed by a measured profile of the
 * stage library (tdp.h):
 *   tdp_prefill_switch_*   Sec. 3.3, Algorithm 1: when to stop launching prefills
 *   tdp_work_stealing_*    Sec. 3.4: keeping the decode batches the same size
 *   tdp_*_intensity, tdp_switch_to_prefill
 *                          Sec. 3.5, Eq. 1 and Eq. 2: when to leave the decode phase
 *   tdp_simulate           Sec. 3.1: the temporally-disaggregated pipeline as a whole
 *
 * Conventions: every pointer is a host pointer; arrays are owned by the caller; functions that
 * return int give 0 (or the documented non-negative answer) on success and TDP_SCHED_EINVAL (-1)
 * on a null pointer, a negative size or an output array that is too small; functions that return
 * double give NaN on bad arguments.  Objects are not thread safe; different objects are independent.
 */
#ifndef TDP_SCHED_H
#define TDP_SCHED_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TDP_SCHED_API __attribute__((visibility("default")))
#define TDP_SCHED_EINVAL (-1)
#define TDP_SCHED_EABORT (-2) /* an executor callback returned nonzero: the run stopped there */

TDP_SCHED_API int tdp_sched_abi_version(void); /* 1 */

/* ---- Sec. 3.3, Algorithm 1: prefill-to-decode switch --------------------------------------------
 * kvUsage[p] = predicted KV-cache occupancy, in tokens, p decode steps from now, kept for the
 * future points p (default 32, 64, ..., 1024: future_points null).  UpdateUsage adds
 * input_len + p at every future point p <= predict_len; CheckSwitch says "switch to decode" when
 * the largest entry exceeds kv_capacity (tokens). */
typedef struct tdp_prefill_switch tdp_prefill_switch;
TDP_SCHED_API int tdp_prefill_switch_create(int64_t kv_capacity, const int32_t* future_points, int32_t n_points,
                                            tdp_prefill_switch** out);
TDP_SCHED_API void tdp_prefill_switch_destroy(tdp_prefill_switch* s);
TDP_SCHED_API int tdp_prefill_switch_reset(tdp_prefill_switch* s);
TDP_SCHED_API int tdp_prefill_switch_update(tdp_prefill_switch* s, int32_t input_len, int32_t predict_len);
/* copies kvUsage, in future-point order, into usage_out[0..n); n must be at least the number of points;
 * returns the number of points */
TDP_SCHED_API int tdp_prefill_switch_usage(const tdp_prefill_switch* s, int64_t* usage_out, int32_t n);
/* 1 = switch to decode, 0 = remain in prefill */
TDP_SCHED_API int tdp_prefill_switch_check(const tdp_prefill_switch* s);

/* ---- Sec. 3.4: inter-batch work stealing ---------------------------------------------------------
 * n_batches = number of pipeline stages = length of the sliding window.  The requests are divided
 * evenly at creation (the first n_requests % n_batches batches get one more).  on_return is called
 * when a batch comes back from the last stage: its finished requests are dropped, the average is
 * ceil(live requests, withheld ones included, / n_batches); a batch above the average gives up its
 * tail to the withheld queue, a batch below it is topped up from that queue first in first out.
 * The new composition is written to ids_out (capacity cap) and its length to *n_out. */
typedef struct tdp_work_stealing tdp_work_stealing;
TDP_SCHED_API int tdp_work_stealing_create(int32_t n_batches, const int64_t* request_ids, int32_t n_requests,
                                           tdp_work_stealing** out);
TDP_SCHED_API void tdp_work_stealing_destroy(tdp_work_stealing* w);
TDP_SCHED_API int tdp_work_stealing_batch(const tdp_work_stealing* w, int32_t batch, int64_t* ids_out, int32_t cap,
                                          int32_t* n_out);
TDP_SCHED_API int tdp_work_stealing_withheld(const tdp_work_stealing* w, int64_t* ids_out, int32_t cap,
                                             int32_t* n_out);
TDP_SCHED_API int tdp_work_stealing_on_return(tdp_work_stealing* w, int32_t batch, const int64_t* finished_ids,
                                              int32_t n_finished, int64_t* ids_out, int32_t cap, int32_t* n_out);

/* ---- Sec. 3.5: spatial-temporal intensity comparison ---------------------------------------------
 * A profile is n points (x[i], ms[i]) with x ascending: x = decode batch size (or prefill tokens),
 * ms = time of one stage pass.  Between points the time is interpolated linearly, below x[0] it is
 * ms[0], above x[n-1] it grows in proportion to x. */
TDP_SCHED_API double tdp_profile_time(const double* x, const double* ms, int32_t n, double at);
/* Eq. 1: Achieved / Peak with Achieved(b) = b / time(b) and Peak = the largest x[i] / ms[i] */
TDP_SCHED_API double tdp_spatial_intensity(const double* x, const double* ms, int32_t n, double batch);
/* Eq. 2: 1 - bubble / total; bubble = max(0, longest pending prefill - decode_ms); total = sum of the
 * pending prefills + bubble (+ n_batches * decode_ms when count_decode_steps); 0 with nothing pending */
TDP_SCHED_API double tdp_temporal_intensity(const double* pending_prefill_ms, int32_t n_pending, double decode_ms,
                                            int32_t n_batches, int32_t count_decode_steps);
/* 1 = switch to prefill (spatial < temporal), 0 = keep decoding */
TDP_SCHED_API int tdp_switch_to_prefill(const double* x, const double* ms, int32_t n, double batch,
                                        const double* pending_prefill_ms, int32_t n_pending, double decode_ms,
                                        int32_t n_batches, int32_t count_decode_steps);

/* ---- Sec. 3.1: the pipeline as a whole, simulated -------------------------------------------------
 * Offline run: request r has input_len[r] prompt tokens, generates output_len[r] >= 1 tokens (the
 * first one in its prefill) and is predicted to generate predict_len[r].  Stage times come from the
 * two profiles.  A batch visits the stages in order, a stage runs one batch at a time, a decode
 * batch re-enters stage 0 when its previous step has left the last stage.  Phases alternate:
 * prefill batches (first come first served, up to prefill_token_budget tokens, at least one prompt)
 * are launched until Algorithm 1 says stop (greedy_prefill = 0: until the prompts no longer fit);
 * the decode phase runs n_stages batches with or without work stealing and ends by the intensity
 * rule (intensity_switch = 0: when every running request is done).  A request that does not fit
 * any more during decode is recomputed later (its generated tokens join its prompt).
 * Phase switches are compact (Sec. 3.1): after a switch to prefill is decided the prefill batches enter stage 0
 * behind the decode steps still in flight (the bubble is the mismatch of step times, Sec. 3.5), and a decode
 * batch starts as soon as stage 0 is free and each of its requests has the token its prefill produced.
 * Events, in the order the scheduler handles them (times are not monotone across a switch to prefill, where
 * the steps in flight return while the first prefills are under way): kind 0 = prefill batch left the pipeline (a = requests, b =
 * tokens), 1 = decode batch returned (a = batch index, b = size it is resubmitted with), 2 = switch
 * to prefill decided (a = batch size, b = pending prefill batches).  At most events_cap events are
 * written; result->n_events is the number that occurred. */
typedef struct {
  int32_t n_stages;
  int64_t kv_capacity; /* tokens */
  int32_t prefill_token_budget;
  int32_t greedy_prefill, work_stealing, intensity_switch, count_decode_steps;
} tdp_sim_config;
typedef struct {
  double total_ms, busy_ms; /* busy: summed over stages */
  int64_t generated_tokens, prefill_tokens, peak_kv_tokens, n_events;
  int32_t phase_switches, recomputes;
} tdp_sim_result;
typedef struct {
  int32_t kind;
  double time_ms;
  int64_t a, b;
} tdp_sim_event;
TDP_SCHED_API int tdp_simulate(const tdp_sim_config* cfg, const int32_t* input_len, const int32_t* output_len,
                               const int32_t* predict_len, int64_t n_requests, const double* decode_x,
                               const double* decode_ms, int32_t n_decode, const double* prefill_x,
                               const double* prefill_ms, int32_t n_prefill, tdp_sim_result* result,
                               tdp_sim_event* events, int64_t events_cap);

/* ---- the same run with the work done for real ----------------------------------------------------
 * tdp_simulate_exec takes the same decisions in the same order (the pipeline clock still comes from
 * the two profiles) and, at every event, calls the executor so that a worker can run the batch the
 * event stands for: this is how the decisions of Sec. 3.3 - 3.5 drive the stage library (tdp.h) on
 * one GPU.  Callbacks run on the calling thread, between decisions; any of them may be null; a
 * nonzero return stops the run (TDP_SCHED_EABORT).  exec = null is tdp_simulate.
 *   prefill(user, ids, input_len, n)   a prefill batch, in packing order; input_len[i] tokens of request
 *                                      ids[i] are to be prefilled from position 0 (for a request that was
 *                                      evicted earlier: its prompt plus everything it had generated) and
 *                                      yield its next token
 *   decode(user, batch, ids, context, n)  one decode step of pipeline batch `batch`: request ids[i] holds
 *                                      context[i] tokens in the cache, its newest token goes in at that
 *                                      position and the step yields the next one
 *   release(user, ids, n, reason)      the requests leave the cache: reason 0 = finished, 1 = evicted
 *                                      (memory overflow: they will be prefilled again later) */
typedef struct {
  void* user;
  int (*prefill)(void* user, const int64_t* ids, const int32_t* input_len, int32_t n);
  int (*decode)(void* user, int32_t batch, const int64_t* ids, const int32_t* context, int32_t n);
  int (*release)(void* user, const int64_t* ids, int32_t n, int32_t reason);
} tdp_sim_executor;
TDP_SCHED_API int tdp_simulate_exec(const tdp_sim_config* cfg, const int32_t* input_len, const int32_t* output_len,
                                    const int32_t* predict_len, int64_t n_requests, const double* decode_x,
                                    const double* decode_ms, int32_t n_decode, const double* prefill_x,
                                    const double* prefill_ms, int32_t n_prefill, tdp_sim_result* result,
                                    tdp_sim_event* events, int64_t events_cap, const tdp_sim_executor* exec);

#ifdef __cplusplus
}
#endif
#endif
