/*
 * ag_sched.h - C ABI of the host-side scheduling layer that sits on top of the attention kernels (ag.h):
 *   - the TPOT-driven feedback controller (paper Sec. III-B, Algorithm 1), which moves the decode
 *     reservation R_min and the resume-prefill token budget B_prefill against the measured time per
 *     decode step;
 *   - the table of pre-established partitions (paper Sec. III-C, "Green Context allocation and
 *     rebinding"): pairs of CU-masked streams created once, a decode stream on the first r CUs of every
 *     XCD and a prefill stream on the complement, between which a rebinding is a table lookup.
 *
 * Everything here runs on the host.  Objects are created and destroyed by the caller through the functions
 * below; each object carries its own mutex, so the decode thread, the prefill thread and the scheduler
 * (paper Sec. III-C, two submission threads plus the scheduler) may call into one object concurrently.
 * Functions return an ag_status (ag.h) unless stated; messages through ag_last_error().
 *
 * Units: times are microseconds (double).  R counts allocation units; on MI355X one unit is one CU in
 * every XCD (8 CUs), so S = 32 units cover the 256 CUs.
 */
#ifndef AG_SCHED_H
#define AG_SCHED_H

#include "ag.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Request classes (paper Sec. I, Fig. 1) and the two queues of Algorithm 1. */
typedef enum { AG_REQ_DECODE = 0, AG_REQ_RESUME = 1, AG_REQ_COLD = 2 } ag_req_type;
typedef enum { AG_QUEUE_DECODE = 0, AG_QUEUE_PREFILL = 1 } ag_queue;

/*
 * Parameters of Algorithm 1.  The listing uses B_min, B_max and R_base without declaring them and the paper
 * gives no value for any constant; all are the caller's choice.  Requirements (else AG_ERR_INVALID_ARG):
 * 0 < r_base <= r_init <= S, 0 <= b_min <= b_init <= b_max, delta_r >= 0, delta_b >= 0,
 * theta_low_us <= theta_high_us.
 */
typedef struct ag_ctl_params {
    int32_t S;              /* allocation units on the device */
    int32_t r_base;         /* floor of the decode reservation */
    int32_t r_init;         /* R_min at start */
    int32_t b_init;         /* B_prefill at start (tokens) */
    int32_t delta_r;        /* step of R_min per control interval */
    int32_t delta_b;        /* step of B_prefill per control interval (tokens) */
    int32_t b_min, b_max;   /* range of B_prefill */
    double  theta_low_us;   /* below this TPOT_step the controller relaxes */
    double  theta_high_us;  /* above this TPOT_step the controller protects decode */
} ag_ctl_params;

typedef struct ag_ctl_state {
    int32_t r_min;          /* decode reservation, units */
    int32_t b_prefill;      /* resume-prefill token budget */
    double  tpot_us;        /* TPOT_step of the last closed interval; NaN if it held no decode step */
    int64_t intervals;      /* control intervals closed so far */
    int64_t raised, lowered;/* intervals that raised / lowered R_min's side of the rule (protect / relax) */
} ag_ctl_state;

typedef struct ag_ctl ag_ctl;

AG_API ag_status ag_ctl_create(const ag_ctl_params* params, ag_ctl** out);
AG_API ag_status ag_ctl_destroy(ag_ctl* ctl);

/* The decode thread reports one completed decode step of the given duration (adds to dL, counts in dK). */
AG_API ag_status ag_ctl_record_decode(ag_ctl* ctl, double step_us);

/*
 * Closes one control interval (the loop body of Algorithm 1 up to the classification): TPOT_step = dL / dK
 * over the steps recorded since the last tick; above theta_high, B_prefill drops by delta_b (not below
 * b_min) and R_min rises by delta_r (not above S); below theta_low the opposite (not above b_max, not below
 * r_base); both comparisons are strict.  An interval without a decode step changes nothing (the paper leaves
 * 0/0 open).  The caller provides the cadence: call it every control interval.  state_out may be NULL.
 */
AG_API ag_status ag_ctl_tick(ag_ctl* ctl, ag_ctl_state* state_out);
AG_API ag_status ag_ctl_get(ag_ctl* ctl, ag_ctl_state* state_out);

/*
 * Queue for a request under the current B_prefill: decodes, and resume prefills of at most B_prefill
 * tokens, go to the decode queue; longer resume prefills and every cold prefill (paper Sec. III-A: cold
 * prefills have their own queue) go to the prefill queue.  Returns an ag_queue, or AG_ERR_INVALID_ARG (< 0).
 */
AG_API int32_t ag_ctl_classify(ag_ctl* ctl, int32_t req_type, int32_t len_tokens);

/*
 * The rebinding rule (paper Sec. III-C): partitions exist at g, 2g, ... units and at S; returns the decode
 * size of the smallest one with at least r_min units (a 37 % target takes the 40 % partition), S if none
 * is large enough, or AG_ERR_INVALID_ARG (< 0) unless 0 < g <= S.  Pure host arithmetic.
 */
AG_API int32_t ag_partition_level_for(int32_t S, int32_t g, int32_t r_min);

/*
 * Table of pre-established partitions on the current device.  Entry i (0-based) gives decode the first
 * (i+1)*g CUs of every XCD (the last entry all of them) and prefill the remaining CUs; both are CU-masked
 * streams of default priority created once here.  The last entry has no prefill stream (NULL): with the
 * whole device reserved for decode, prefill launches must wait.  Creating streams is the expensive part
 * (the paper creates its contexts offline for that reason); a rebinding afterwards is ag_slots_bind, a
 * lookup.  Work already enqueued on a previously bound stream keeps the CUs it was launched with until it
 * finishes: the new partition holds for launches made after the call.
 */
typedef struct ag_slots ag_slots;

AG_API ag_status ag_slots_create(int32_t g_units, ag_slots** out);
AG_API ag_status ag_slots_destroy(ag_slots* slots);     /* synchronises and destroys the streams */
AG_API int32_t   ag_slots_count(const ag_slots* slots);  /* number of entries, or < 0 */
AG_API int32_t   ag_slots_units(const ag_slots* slots);  /* S: CUs per XCD, or < 0 */
/* Entry `index`: decode size in units, and the two streams (hipStream_t; prefill NULL in the last entry). */
AG_API ag_status ag_slots_get(const ag_slots* slots, int32_t index, int32_t* decode_units,
                              void** decode_stream, void** prefill_stream);
/* Selects the entry ag_partition_level_for(S, g, r_min) names, remembers it as current, returns its index. */
AG_API ag_status ag_slots_bind(ag_slots* slots, int32_t r_min, int32_t* index_out);
AG_API int32_t   ag_slots_current(const ag_slots* slots);

#ifdef __cplusplus
}
#endif
#endif /* AG_SCHED_H */
