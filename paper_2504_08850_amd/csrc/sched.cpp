// Online half of the two-level scheduler (paper Sec. 5.3): a circular queue of
// the exit layers of the last Q tokens and, per layer, the number of queued
// exits within `radius` of it.  Host-side integer bookkeeping; the caller owns
// the state, nothing is allocated.
#include "../../include/specee.h"

namespace {

void bump(specee_sched *s, int layer, int delta) {
    int lo = layer - s->radius, hi = layer + s->radius;
    if (lo < 0) lo = 0;
    if (hi > s->L - 1) hi = s->L - 1;
    for (int i = lo; i <= hi; ++i) s->counter[i] += delta;
}

}  // namespace

extern "C" {

int specee_sched_init(specee_sched *s, int L, int Q, int radius) {
    if (!s || L < 1 || L > SPECEE_SCHED_MAXL || Q < 1 || Q > SPECEE_SCHED_MAXQ || radius < 0) return SPECEE_EINVAL;
    s->L = L;
    s->Q = Q;
    s->radius = radius;
    s->filled = 0;
    s->head = 0;
    for (int i = 0; i < SPECEE_SCHED_MAXQ; ++i) s->queue[i] = -1;
    for (int i = 0; i < SPECEE_SCHED_MAXL; ++i) s->counter[i] = 0;
    return SPECEE_OK;
}

int specee_sched_push(specee_sched *s, int exit_layer) {
    if (!s || exit_layer < 0 || exit_layer >= s->L) return SPECEE_EINVAL;
    if (s->filled == s->Q) {
        bump(s, s->queue[s->head], -1);  // the oldest entry leaves the window
    } else {
        ++s->filled;
    }
    s->queue[s->head] = exit_layer;
    bump(s, exit_layer, +1);
    s->head = (s->head + 1) % s->Q;
    return SPECEE_OK;
}

int specee_sched_active(const specee_sched *s, const int32_t *offline_mask, int32_t *active) {
    if (!s || !active) return SPECEE_EINVAL;
    int n = 0;
    for (int i = 0; i < s->L; ++i) {
        active[i] = (s->counter[i] > 0 || (offline_mask && offline_mask[i] != 0)) ? 1 : 0;
        n += active[i];
    }
    return n;
}

}  // extern "C"
