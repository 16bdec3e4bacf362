// Host-side bookkeeping of BSP / SSP / ASP application of sufficient factors
// (Section 4, "SSP-SFB"; Eq. (1) of Section 5).  Counters only: see sfb_ssp.h.
#include "../../include/sfb_ssp.h"
#include "../../include/sfb.h"

#include <new>
#include <vector>

struct sfb_ssp {
    int32_t P;
    int32_t s;                       // < 0: unbounded
    std::vector<int64_t> clock;      // t_p
    std::vector<int64_t> arrived;    // [p][q] sets of q that have reached p
    std::vector<int64_t> applied;    // [p][q] tau_p^q
    int64_t max_stale;
};

namespace {
inline bool bad(const sfb_ssp* h, int32_t p) { return !h || p < 0 || p >= h->P; }
inline int64_t& at(std::vector<int64_t>& v, const sfb_ssp* h, int32_t p, int32_t q) { return v[(size_t)p * h->P + q]; }
inline int64_t at(const std::vector<int64_t>& v, const sfb_ssp* h, int32_t p, int32_t q)
{
    return v[(size_t)p * h->P + q];
}
}  // namespace

extern "C" {

int sfb_ssp_create(sfb_ssp** out, int32_t P, int32_t s)
{
    if (!out || P < 1) return SFB_EINVAL;
    sfb_ssp* h = new (std::nothrow) sfb_ssp;
    if (!h) return SFB_EINVAL;
    h->P = P;
    h->s = s;
    h->clock.assign((size_t)P, 0);
    h->arrived.assign((size_t)P * P, 0);
    h->applied.assign((size_t)P * P, 0);
    h->max_stale = 0;
    *out = h;
    return SFB_OK;
}

int sfb_ssp_destroy(sfb_ssp* h)
{
    if (!h) return SFB_EINVAL;
    delete h;
    return SFB_OK;
}

int sfb_ssp_can_compute(const sfb_ssp* h, int32_t p)
{
    if (bad(h, p)) return SFB_EINVAL;
    if (h->s < 0) return 1;
    for (int32_t q = 0; q < h->P; ++q)
        if (q != p && h->clock[p] - at(h->applied, h, p, q) > h->s) return 0;
    return 1;
}

int64_t sfb_ssp_computed(sfb_ssp* h, int32_t p)
{
    if (bad(h, p)) return SFB_EINVAL;
    if (sfb_ssp_can_compute(h, p) != 1) return SFB_EINVAL;
    for (int32_t q = 0; q < h->P; ++q) {
        if (q == p) continue;
        const int64_t stale = h->clock[p] - at(h->applied, h, p, q);
        if (stale > h->max_stale) h->max_stale = stale;
    }
    return h->clock[p]++;
}

int64_t sfb_ssp_delivered(sfb_ssp* h, int32_t p, int32_t q)
{
    if (bad(h, p) || bad(h, q) || p == q) return SFB_EINVAL;
    int64_t& a = at(h->arrived, h, p, q);
    if (a >= h->clock[q]) return SFB_EINVAL;   // q has not produced that set yet
    return a++;
}

int sfb_ssp_pop_apply(sfb_ssp* h, int32_t p, int32_t* q_out, int64_t* t_out)
{
    if (bad(h, p) || !q_out || !t_out) return SFB_EINVAL;
    int32_t best_q = -1;
    int64_t best_t = 0;
    for (int32_t q = 0; q < h->P; ++q) {
        if (q == p) continue;
        const int64_t t = at(h->applied, h, p, q);           // next set of q to apply at p
        if (t >= at(h->arrived, h, p, q)) continue;          // not here yet
        if (t >= h->clock[p]) continue;                      // ahead of p's own clock: held back
        if (best_q < 0 || t < best_t) {
            best_q = q;
            best_t = t;
        }
    }
    if (best_q < 0) return 0;
    at(h->applied, h, p, best_q)++;
    *q_out = best_q;
    *t_out = best_t;
    return 1;
}

int64_t sfb_ssp_clock(const sfb_ssp* h, int32_t p) { return bad(h, p) ? (int64_t)SFB_EINVAL : h->clock[p]; }

int64_t sfb_ssp_tau(const sfb_ssp* h, int32_t p, int32_t q)
{
    if (bad(h, p) || bad(h, q)) return SFB_EINVAL;
    return p == q ? h->clock[p] : at(h->applied, h, p, q);
}

int64_t sfb_ssp_arrived(const sfb_ssp* h, int32_t p, int32_t q)
{
    if (bad(h, p) || bad(h, q)) return SFB_EINVAL;
    return p == q ? h->clock[p] : at(h->arrived, h, p, q);
}

int64_t sfb_ssp_max_staleness_seen(const sfb_ssp* h) { return h ? h->max_stale : (int64_t)SFB_EINVAL; }

}  // extern "C"
