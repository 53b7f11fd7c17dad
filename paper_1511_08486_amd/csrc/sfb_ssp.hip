// Stale-synchronous SFB on one device (Section 4.1 "SSP-SFB", local update rule of Section 5):
// host-side bookkeeping of the workers' clocks on top of the library's own entry points.
// All arithmetic runs in the kernels behind sfb_compute_factors_worker (a worker's factors at
// its own replica) and sfb_reconstruct_apply_worker (a replica applying one sender's factors).
#include <hip/hip_runtime.h>

#include <new>
#include <vector>

#include "../../include/sfb.h"

struct sfb_ssp {
    sfb_ctx* ctx;
    int32_t P, B, staleness, slots;
    int64_t J, D, ldw, ldu, ldv;
    size_t v_elem;                       // bytes per element of V
    std::vector<float*> W;               // P replicas
    float* U_ring;
    char* V_ring;
    std::vector<int32_t> t;              // [P]   iterations completed
    std::vector<int32_t> tau;            // [P][P] sets of q applied at replica p
    std::vector<float> eta;              // [slots][P] step size of the set held in that slot
    std::vector<uint8_t> sends;          // [P][P] sends[q * P + p] != 0: worker q's factors go to replica p
    sfb_status broken;                   // a launch failed after part of an event was enqueued: the replicas and
                                         // the clocks no longer describe the same state, every later event is refused
};

namespace {

float* u_slot(const sfb_ssp* s, int32_t iter) {
    return s->U_ring + (size_t)(iter % s->slots) * (size_t)s->P * s->B * (size_t)s->ldu;
}
void* v_slot(const sfb_ssp* s, int32_t iter) {
    return s->V_ring + (size_t)(iter % s->slots) * (size_t)s->P * s->B * (size_t)s->ldv * s->v_elem;
}

}  // namespace

extern "C" {

sfb_status sfb_ssp_create(sfb_ssp** out, sfb_ctx* ctx, int32_t staleness, float* const* W_replicas, int64_t ldw,
                          float* U_ring, int64_t ldu, void* V_ring, int64_t ldv, int32_t ring_slots) {
    if (!out) return SFB_EINVAL;
    *out = nullptr;
    if (!ctx || !W_replicas || !U_ring || !V_ring || staleness < 0) return SFB_EINVAL;
    int64_t J = 0, D = 0;
    int32_t P = 0, B = 0, dtype = 0;
    sfb_status st = sfb_shape(ctx, &J, &D, &P, &B, &dtype);
    if (st != SFB_OK) return st;
    if (ldw < D || ldu < J || ldv < D) return SFB_ESHAPE;
    if ((int64_t)ring_slots < 2 * (int64_t)staleness + 2) return SFB_ESHAPE;
    for (int32_t p = 0; p < P; ++p)
        if (!W_replicas[p]) return SFB_EINVAL;
    sfb_ssp* s = new (std::nothrow) sfb_ssp();
    if (!s) return SFB_EINVAL;
    s->ctx = ctx;
    s->P = P; s->B = B; s->staleness = staleness; s->slots = ring_slots;
    s->J = J; s->D = D; s->ldw = ldw; s->ldu = ldu; s->ldv = ldv;
    s->v_elem = dtype == SFB_BF16 ? 2 : 4;
    s->W.assign(W_replicas, W_replicas + P);
    s->U_ring = U_ring;
    s->V_ring = (char*)V_ring;
    s->t.assign(P, 0);
    s->tau.assign((size_t)P * P, 0);
    s->eta.assign((size_t)ring_slots * P, 0.f);
    s->sends.assign((size_t)P * P, 1);   // full broadcast
    s->broken = SFB_OK;
    *out = s;
    return SFB_OK;
}

void sfb_ssp_destroy(sfb_ssp* s) { delete s; }

sfb_status sfb_ssp_worker_step(sfb_ssp* s, int32_t p, const sfb_batch* batch_p, const int32_t* y_p, float eta,
                               float* loss, int32_t* blocked) {
    if (!s || !blocked) return SFB_EINVAL;
    if (s->broken != SFB_OK) return s->broken;
    if (p < 0 || p >= s->P) return SFB_ESHAPE;
    const int32_t P = s->P, c = s->t[p];
    for (int32_t q = 0; q < P; ++q) {
        if (q != p && s->sends[(size_t)q * P + p] && c - s->tau[(size_t)p * P + q] > s->staleness) {
            *blocked = 1;            // some sender q is more than `staleness` iterations behind from p's point of view
            return SFB_OK;
        }
    }
    // the slot of iteration c is free once every receiver has applied iteration c - slots of worker p
    for (int32_t r = 0; r < P; ++r) {
        if (r != p && s->sends[(size_t)p * P + r] && c - s->tau[(size_t)r * P + p] >= s->slots) {
            *blocked = 2;            // send queue full
            return SFB_OK;
        }
    }
    *blocked = 0;
    float* U = u_slot(s, c);
    void* V = v_slot(s, c);
    sfb_status st = sfb_compute_factors_worker(s->ctx, s->W[p], s->ldw, batch_p, y_p, p, U, s->ldu, V, s->ldv, loss);
    // validation errors come back before anything is launched; a failed launch may have left part of the
    // factors in the ring slot
    if (st != SFB_OK) return st == SFB_EHIP ? (s->broken = st) : st;
    float scale;                              // mini-batch mean inside a worker (Section 3)
    (void)sfb_default_scale(s->ctx, &scale);
    st = sfb_reconstruct_apply_worker(s->ctx, s->W[p], s->ldw, U, s->ldu, V, s->ldv, p, eta, scale);
    if (st != SFB_OK) return s->broken = st;  // the factors are in the ring but the worker's own update is not applied
    s->eta[(size_t)(c % s->slots) * P + p] = eta;
    s->t[p] = c + 1;
    s->tau[(size_t)p * P + p] = c + 1;
    return SFB_OK;
}

sfb_status sfb_ssp_deliver(sfb_ssp* s, int32_t p, int32_t q, int32_t count) {
    if (!s) return SFB_EINVAL;
    if (s->broken != SFB_OK) return s->broken;
    if (p < 0 || p >= s->P || q < 0 || q >= s->P) return SFB_ESHAPE;
    if (p == q || count < 0) return SFB_EINVAL;
    const int32_t P = s->P;
    if (!s->sends[(size_t)q * P + p]) return SFB_EINVAL;   // q does not broadcast to p
    const int32_t have = s->tau[(size_t)p * P + q];
    if (have + count > s->t[q]) return SFB_EINVAL;     // q has not produced that many
    if (have + count > s->t[p]) return SFB_EINVAL;     // no fast-forward
    float scale;
    (void)sfb_default_scale(s->ctx, &scale);
    for (int32_t it = have; it < have + count; ++it) {
        sfb_status st = sfb_reconstruct_apply_worker(s->ctx, s->W[p], s->ldw, u_slot(s, it), s->ldu, v_slot(s, it),
                                                     s->ldv, q, s->eta[(size_t)(it % s->slots) * P + q], scale);
        if (st != SFB_OK) return s->broken = st;   // sets before `it` are applied and counted, this one is not
        s->tau[(size_t)p * P + q] = it + 1;
    }
    return SFB_OK;
}

sfb_status sfb_ssp_set_receivers(sfb_ssp* s, const uint8_t* sends) {
    if (!s || !sends) return SFB_EINVAL;
    // only before anything has been produced: the clocks assume one topology throughout
    for (int32_t p = 0; p < s->P; ++p)
        if (s->t[p] != 0) return SFB_EINVAL;
    s->sends.assign(sends, sends + (size_t)s->P * s->P);
    return SFB_OK;
}

sfb_status sfb_halton_receivers(int32_t P, int32_t Q, uint8_t* sends) {
    if (P < 1 || Q < 0 || !sends) return SFB_EINVAL;
    for (size_t i = 0; i < (size_t)P * P; ++i) sends[i] = 0;
    // offsets floor(P * num / level) for level = 2, 4, 8, ... and odd num ascending (the order
    // Section 4.3 prints: P/2, P/4, 3P/4, P/8, 3P/8, ...); zero and repeated offsets are skipped
    std::vector<int32_t> offs;
    for (int64_t level = 2; (int32_t)offs.size() < Q && level <= 2 * (int64_t)P; level *= 2) {
        for (int64_t num = 1; num < level && (int32_t)offs.size() < Q; num += 2) {
            const int32_t off = (int32_t)(((int64_t)P * num / level) % P);
            bool seen = off == 0;
            for (int32_t o : offs) seen = seen || o == off;
            if (!seen) offs.push_back(off);
        }
    }
    for (int32_t p = 0; p < P; ++p)
        for (int32_t o : offs) sends[(size_t)p * P + (p + o) % P] = 1;
    return SFB_OK;
}

sfb_status sfb_ssp_state(const sfb_ssp* s, int32_t* t, int32_t* tau) {
    if (!s) return SFB_EINVAL;
    if (t)
        for (int32_t p = 0; p < s->P; ++p) t[p] = s->t[p];
    if (tau)
        for (size_t i = 0; i < s->tau.size(); ++i) tau[i] = s->tau[i];
    return SFB_OK;
}

}  // extern "C"
