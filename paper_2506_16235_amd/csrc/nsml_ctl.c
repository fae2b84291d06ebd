/*
 * Host side of libnsml: the network-sensing controller (Algorithm 1, Eq. (1)-(3)), the
 * quantization gate (Algorithm 2 Step 1) and the payload geometry.  Plain C, no GPU calls.
 */
#include <math.h>
#include <stddef.h>
#include <string.h>

#include "nsml.h"

const char *nsml_strerror(int code)
{
    switch (code) {
    case NSML_OK:       return "ok";
    case NSML_EINVAL:   return "invalid argument";
    case NSML_ECAP:     return "exceeds the capacity the context was created with";
    case NSML_EHIP:     return "a HIP call failed";
    case NSML_ENOTIMPL: return "not implemented";
    case NSML_ENOMEM:   return "out of host memory";
    case NSML_EINTERNAL: return "internal consistency check failed";
    default:            return "unknown error";
    }
}

int nsml_ctl_default_params(nsml_ctl_params *p)
{
    if (!p) return NSML_EINVAL;
    p->alpha = 0.5;       /* Sec. 4.1, after Eq. (3) */
    p->beta1 = 0.1;
    p->beta2 = 0.01;      /* Sec. 4.1, after Eq. (3) */
    p->floor = 0.005;     /* Eq. (3) */
    p->cap = 1.0;         /* Eq. (3) */
    p->init = 0.01;       /* Algorithm 1 Step 1 */
    p->bdp_frac = 0.9;    /* Eq. (3) */
    p->rtt_excess = 2.0;
    p->tr_q = 0.1;
    p->tr_q4 = 0.01;
    p->tr_d = 0.0;
    p->startup_max = 10;
    p->win_bw = 10;
    p->win_rt = 100;
    p->quant_mode = 0;
    return NSML_OK;
}

int nsml_ctl_init(nsml_ctl_state *s, const nsml_ctl_params *p)
{
    if (!s) return NSML_EINVAL;
    nsml_ctl_params d;
    if (!p) { nsml_ctl_default_params(&d); p = &d; }
    if (p->win_bw < 0 || p->win_bw > NSML_CTL_MAX_WIN || p->win_rt < 0 || p->win_rt > NSML_CTL_MAX_WIN)
        return NSML_EINVAL;
    if (!(p->floor > 0.0) || !(p->cap <= 1.0) || !(p->floor <= p->cap)) return NSML_EINVAL;
    if (!(p->init >= p->floor && p->init <= p->cap)) return NSML_EINVAL;
    if (!(p->alpha > 0.0 && p->alpha < 1.0) || !(p->beta1 >= 0.0) || !(p->beta2 >= 0.0)) return NSML_EINVAL;
    if (p->quant_mode < 0 || p->quant_mode > 2 || p->startup_max < 0) return NSML_EINVAL;
    memset(s, 0, sizeof(*s));
    s->p = *p;
    s->ratio = p->init;
    s->phase = 0;
    return NSML_OK;
}

/* max (want_max) or min over the newest `win` entries of a ring that has seen `count` pushes */
static double ring_extreme(const double *ring, int64_t count, int win, int want_max)
{
    int64_t have = count < NSML_CTL_MAX_WIN ? count : NSML_CTL_MAX_WIN;
    int64_t take = win < have ? win : have;
    double best = ring[(count - 1) % NSML_CTL_MAX_WIN];
    for (int64_t i = 1; i < take; ++i) {
        double x = ring[(count - 1 - i) % NSML_CTL_MAX_WIN];
        if (want_max ? x > best : x < best) best = x;
    }
    return best;
}

int nsml_choose_ratio(nsml_ctl_state *s, double last_payload_bytes, double last_tx_seconds,
                      double dense_bytes, double last_l2norm, double *ratio_out, int *bits_out)
{
    (void)dense_bytes;
    if (!s || !ratio_out || !bits_out) return NSML_EINVAL;
    const nsml_ctl_params *p = &s->p;

    if (last_payload_bytes > 0.0 && last_tx_seconds > 0.0) {
        /* Eq. (1): estimated bandwidth of the interval that just ended */
        const double ebb = last_payload_bytes / last_tx_seconds;
        s->ebb[s->count % NSML_CTL_MAX_WIN] = ebb;
        s->rtt[s->count % NSML_CTL_MAX_WIN] = last_tx_seconds;
        if (s->count == 0 || ebb > s->all_max_ebb) s->all_max_ebb = ebb;
        if (s->count == 0 || last_tx_seconds < s->all_min_rtt) s->all_min_rtt = last_tx_seconds;
        s->count += 1;
        /* Algorithm 1 Step 2: BtlBw = max EBB, RTprop = min RTT */
        s->btlbw  = p->win_bw > 0 ? ring_extreme(s->ebb, s->count, p->win_bw, 1) : s->all_max_ebb;
        s->rtprop = p->win_rt > 0 ? ring_extreme(s->rtt, s->count, p->win_rt, 0) : s->all_min_rtt;
        /* Eq. (2) */
        s->bdp = s->btlbw * s->rtprop;

        if (s->phase == 0) {
            /* Algorithm 1 Step 1: ramp until excessive RTT, a step limit, or the cap */
            const int excessive = last_tx_seconds > p->rtt_excess * s->rtprop;
            if (excessive || s->startup_steps >= p->startup_max || s->ratio >= p->cap) {
                s->phase = 1;
            } else {
                s->ratio = fmin(p->cap, s->ratio + p->beta1);
                s->startup_steps += 1;
            }
        }
        if (s->phase == 1) {
            /* Eq. (3) */
            if (last_payload_bytes > p->bdp_frac * s->bdp)
                s->ratio = fmax(p->floor, s->ratio * p->alpha);
            else
                s->ratio = fmin(p->cap, s->ratio + p->beta2);
        }
    }

    /* Algorithm 2 Step 1: below tr_q, and if the gradient carries enough signal, send narrower
     * values and let top-k keep twice as many of them */
    double r = s->ratio;
    int bits = 32;
    if (p->quant_mode != 2 && s->ratio < p->tr_q && (last_l2norm < 0.0 || last_l2norm > p->tr_d)) {
        bits = p->quant_mode == 1 ? 16 : (s->ratio < p->tr_q4 ? 4 : 8);
        r = fmin(p->cap, 2.0 * s->ratio);
    }
    *ratio_out = r;
    *bits_out = bits;
    return NSML_OK;
}

/* Algorithm 2 Step 3: how many entries top_k(grads, ratio) keeps in a bucket of n_b. */
static uint64_t survivors(double ratio, uint64_t n_b)
{
    if (n_b == 0) return 0;
    const double want = ceil(ratio * (double)n_b);
    if (want < 1.0) return 1;
    if (want >= (double)n_b) return n_b;
    return (uint64_t)want;
}

int nsml_payload_layout(const uint64_t *bucket_off, uint32_t B, double ratio, int bits,
                        uint32_t chunk, uint64_t *k_b, uint64_t *K, uint64_t *val_bytes,
                        uint64_t *n_scales)
{
    if (!bucket_off || B == 0 || chunk == 0 || chunk % 8 != 0) return NSML_EINVAL;
    if (!(ratio > 0.0 && ratio <= 1.0)) return NSML_EINVAL;
    if (bits != 4 && bits != 8 && bits != 16 && bits != 32) return NSML_EINVAL;
    uint64_t tk = 0, tv = 0, ts = 0;
    for (uint32_t b = 0; b < B; ++b) {
        if (bucket_off[b + 1] < bucket_off[b]) return NSML_EINVAL;
        const uint64_t nb = bucket_off[b + 1] - bucket_off[b];
        if (nb > 0xFFFFFFFFull) return NSML_EINVAL;
        const uint64_t k = survivors(ratio, nb);
        if (k_b) k_b[b] = k;
        tk += k;
        tv += bits == 32 ? 4 * k : bits == 16 ? 2 * k : bits == 8 ? k : (k + 1) / 2;
        if (bits <= 8) ts += (k + chunk - 1) / chunk;
    }
    if (K) *K = tk;
    if (val_bytes) *val_bytes = tv;
    if (n_scales) *n_scales = ts;
    return NSML_OK;
}
