/*
 * sfb_ssp.h - bookkeeping of the consistency models under which sufficient
 * factors (SFs) are applied: BSP-SFB, SSP-SFB and ASP-SFB (Section 4, "SSP-SFB"
 * paragraph; the local update rule is Eq. (1) of Section 5).
 *
 * P workers each hold a replica of W.  Worker p computes its SF sets one after
 * the other (set t = 0, 1, ... is computed at its own replica as it stands),
 * applies each of its own sets at once, and applies the sets of a peer q in the
 * order q produced them, as they arrive.  This object only COUNTS; it moves no
 * data and launches no kernel.  The caller computes and applies SF sets with
 * sfb_compute_sf / sfb_apply (sfb.h) and tells this object what happened:
 *
 *   t_p        number of SF sets worker p has computed            (sfb_ssp_clock)
 *   tau_p^q    number of SF sets of q that p has applied          (sfb_ssp_tau)
 *
 * Rules enforced (in the paper's notation, with its 1-based iteration c = t_p + 1):
 *   - staleness: p may compute its next set only while t_p - tau_p^q <= s for
 *     every peer q (otherwise it pauses); s = 0 is BSP, s < 0 means unbounded
 *     (ASP);
 *   - no fast-forward: p applies set t of q only once it has itself computed
 *     set t, i.e. tau_p^q <= t_p always (the second condition of Eq. (1));
 *   - channels are FIFO: the sets of q reach p in the order q produced them.
 *
 * All functions are host-only, thread-compatible (one thread at a time per
 * object), allocate only in sfb_ssp_create, and return 0 / a count on success
 * or a negative sfb_status (sfb.h): SFB_EINVAL for a null handle, an index out
 * of range or an event that the rules above do not allow.
 */
#ifndef SFB_SSP_H
#define SFB_SSP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sfb_ssp sfb_ssp;

/* P >= 1 workers; staleness bound s >= 0, or s < 0 for none (ASP). */
int sfb_ssp_create(sfb_ssp** out, int32_t P, int32_t s);
int sfb_ssp_destroy(sfb_ssp* h);

/* 1 if worker p may compute its next SF set now, 0 if it has to pause. */
int sfb_ssp_can_compute(const sfb_ssp* h, int32_t p);
/* Worker p has computed (and applied to its own replica) its next SF set.
 * Returns the index t of that set (>= 0); SFB_EINVAL if p had to pause. */
int64_t sfb_ssp_computed(sfb_ssp* h, int32_t p);

/* The transport reports that the next SF set of q (in q's order) has reached p.
 * Returns its index t; SFB_EINVAL if q has not produced another set yet. */
int64_t sfb_ssp_delivered(sfb_ssp* h, int32_t p, int32_t q);

/* The next SF set worker p has to apply now: among the peers with a set that
 * has arrived, is not applied yet and is not ahead of p's own clock, the one
 * with the smallest (t, q).  Returns 1 and writes q, t (the set is then counted
 * as applied: the caller runs sfb_apply on it before asking again), or 0 if
 * there is none. */
int sfb_ssp_pop_apply(sfb_ssp* h, int32_t p, int32_t* q, int64_t* t);

/* Counters. */
int64_t sfb_ssp_clock(const sfb_ssp* h, int32_t p);               /* t_p */
int64_t sfb_ssp_tau(const sfb_ssp* h, int32_t p, int32_t q);      /* tau_p^q (q == p: t_p) */
int64_t sfb_ssp_arrived(const sfb_ssp* h, int32_t p, int32_t q);  /* sets of q that have reached p */
/* Largest t_p - tau_p^q seen at the moment a set was computed, over all p, q. */
int64_t sfb_ssp_max_staleness_seen(const sfb_ssp* h);

#ifdef __cplusplus
}
#endif
#endif /* SFB_SSP_H */
