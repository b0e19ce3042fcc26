/*
 * CPU oracle for scoring candidate schedules of multi-call agentic workflows on a disaggregated
 * prefill/decode cluster.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, serial; only the tests may call it; it shares no code with the
 * HIP path.
 *
 * What is computed, and which passage of the paper each step follows (Section 8.3 "Agentic Request
 * Scheduling"; Appendix "Scheduling Problem Formulation", Formulation for Agentic Request):
 *  - A cluster has prefill instances P and decode instances Q; each decode instance has a finite
 *    token-capacity budget, and instances differ in their serving characteristics.
 *  - A workflow arrives at some time and consists of LLM calls, each with an input and an output
 *    length; a call becomes schedulable only when all of its predecessor calls have completed.
 *  - A plan assigns every call to one prefill and one decode instance and fixes the queue order on every
 *    instance.  Prefill instances process one call at a time; decode instances respect their cumulative
 *    token-capacity limit.
 *  - Every workflow has a committed horizon SLO and a completion time C; the quality of a schedule is
 *    the completion ratio C / SLO, reported as mean, 95th and 99th percentile over the workflows.
 *
 * Readings where the paper is silent (a candidate here is a complete plan: both instance ids and one
 * queue key per call; the paper's policies produce such plans round by round):
 *  - release(k) = max(arrival of k's workflow, completion of every predecessor).
 *  - Prefill of call k on instance p takes pa[p] + pb[p] * in_len[k] microseconds, decode on instance q
 *    takes out_len[k] * (qc[q] + qd[q] * ceil(in_len[k] / 1024)); both are at least 1 (checked by the
 *    caller).  During decode the call holds in_len + out_len tokens of q's budget.
 *  - Queue order: among the calls waiting at an instance the one with the smallest (key, call index)
 *    goes first.  An idle prefill instance starts it at once.  A decode instance admits its first
 *    waiting call as soon as it fits the free budget, and only the first (no overtaking).
 *  - Events that fall on the same instant are applied as: decode completions, prefill completions,
 *    releases, decode admissions, prefill starts - so what is freed at t can be reused at t.
 *  - A call that names no existing prefill instance fails when it is released; one that names no
 *    existing decode instance, or needs more tokens than that instance's whole budget, fails when its
 *    prefill completes.  A failed call counts as completed at that instant (its successors go on), and
 *    its workflow is charged the penalty ratio instead of C / SLO.
 *  - ratio = floor(C * 1000 / SLO) (per mille); percentiles by the nearest-rank rule over the W
 *    workflows (rank ceil(q W / 100)); a workflow is late when C > SLO.
 *
 * Pins (tests/test_agentic_pins.py): a hand-worked three-call example, the critical-path closed form
 * when nothing is contended, the single-server prefix sums in key order, serialisation by the token
 * budget, sweep-line invariants of the per-call record (one prefill at a time per instance, budget
 * never exceeded, precedence, no overtaking of waiting calls).  The dynamics above are a reading of
 * the paper, not printed values: parity unpinned for the choice of rules themselves.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    uint32_t W, K;
    const uint64_t *arrival_us;   /* [W] */
    const uint64_t *slo_us;       /* [W], > 0 */
    const uint32_t *wf;           /* [K] workflow of call k */
    const uint32_t *in_len;       /* [K] >= 1 */
    const uint32_t *out_len;      /* [K] >= 1 */
    const uint32_t *pred_first;   /* [K + 1] */
    const uint32_t *pred;         /* predecessors, each < k and in the same workflow */
    uint32_t P, Q;
    const uint32_t *pa, *pb;      /* [P] */
    const uint32_t *qc, *qd;      /* [Q] */
    const uint32_t *cap;          /* [Q] tokens */
    uint64_t penalty_permille;
} ago_problem;

typedef struct {
    uint64_t sum_ratio_permille;
    uint64_t p95_permille;
    uint64_t p99_permille;
    uint64_t makespan_us;         /* latest completion minus earliest arrival */
    uint32_t n_late;              /* workflows with C > SLO (failed ones included) */
    uint32_t n_failed;            /* workflows with a failed call */
} ago_metrics;

typedef struct {                  /* optional per-call record */
    uint64_t *release_us, *pre_start_us, *pre_end_us, *dec_start_us, *done_us;   /* [K] */
    uint8_t *failed;              /* [K] */
} ago_detail;

enum { BLOCKED, WAIT_PRE, IN_PRE, WAIT_DEC, IN_DEC, DONE };

static int cmp_u64(const void *a, const void *b)
{
    uint64_t x = *(const uint64_t *)a, y = *(const uint64_t *)b;
    return x < y ? -1 : x > y;
}

static uint64_t prefill_time(const ago_problem *p, uint32_t inst, uint32_t k)
{
    return (uint64_t)p->pa[inst] + (uint64_t)p->pb[inst] * p->in_len[k];
}

static uint64_t decode_time(const ago_problem *p, uint32_t inst, uint32_t k)
{
    uint64_t kctx = ((uint64_t)p->in_len[k] + 1023u) / 1024u;
    return (uint64_t)p->out_len[k] * ((uint64_t)p->qc[inst] + (uint64_t)p->qd[inst] * kctx);
}

int ago_eval(const ago_problem *p, const uint16_t *pre_inst, const uint16_t *dec_inst, const uint32_t *key,
             ago_metrics *out, const ago_detail *det)
{
    const uint32_t K = p->K, W = p->W;
    uint8_t *phase = calloc(K, 1), *failed = calloc(K, 1), *wf_failed = calloc(W, 1), *pre_busy = calloc(p->P ? p->P : 1, 1);
    uint64_t *t_event = calloc(K, 8), *done = calloc(K, 8), *used = calloc(p->Q ? p->Q : 1, 8);
    uint64_t *rel = calloc(K, 8), *ps = calloc(K, 8), *pe = calloc(K, 8), *ds = calloc(K, 8), *ratio = calloc(W ? W : 1, 8);
    if (!phase || !failed || !wf_failed || !pre_busy || !t_event || !done || !used || !rel || !ps || !pe || !ds || !ratio)
        return 2;

    for (;;) {
        /* the next instant at which something happens */
        int any = 0;
        uint64_t t = 0;
        for (uint32_t k = 0; k < K; ++k) {
            uint64_t cand;
            if (phase[k] == IN_PRE || phase[k] == IN_DEC) cand = t_event[k];
            else if (phase[k] == BLOCKED) cand = p->arrival_us[p->wf[k]];   /* blocked calls wake up at arrival at the earliest */
            else continue;
            if (phase[k] == BLOCKED) {
                /* only an event if the call could be released then: all predecessors done */
                int ready = 1;
                for (uint32_t i = p->pred_first[k]; i < p->pred_first[k + 1]; ++i) ready = ready && phase[p->pred[i]] == DONE;
                if (!ready) continue;
                for (uint32_t i = p->pred_first[k]; i < p->pred_first[k + 1]; ++i)
                    if (done[p->pred[i]] > cand) cand = done[p->pred[i]];
            }
            if (!any || cand < t) t = cand;
            any = 1;
        }
        if (!any) break;

        /* 1. completions: decode, then prefill */
        for (uint32_t k = 0; k < K; ++k)
            if (phase[k] == IN_DEC && t_event[k] == t) {
                phase[k] = DONE;
                done[k] = t;
                used[dec_inst[k]] -= (uint64_t)p->in_len[k] + p->out_len[k];
            }
        for (uint32_t k = 0; k < K; ++k)
            if (phase[k] == IN_PRE && t_event[k] == t) {
                pre_busy[pre_inst[k]] = 0;
                pe[k] = t;
                uint32_t q = dec_inst[k];
                if (q >= p->Q || (uint64_t)p->in_len[k] + p->out_len[k] > p->cap[q]) {
                    phase[k] = DONE; done[k] = t; failed[k] = 1; wf_failed[p->wf[k]] = 1;
                } else {
                    phase[k] = WAIT_DEC;
                }
            }
        /* 2. releases, in index order (a call that fails here completes at t and may release later calls) */
        for (uint32_t k = 0; k < K; ++k) {
            if (phase[k] != BLOCKED || p->arrival_us[p->wf[k]] > t) continue;
            int ready = 1;
            for (uint32_t i = p->pred_first[k]; i < p->pred_first[k + 1]; ++i) ready = ready && phase[p->pred[i]] == DONE;
            if (!ready) continue;
            rel[k] = t;
            if (pre_inst[k] >= p->P) {
                phase[k] = DONE; done[k] = t; failed[k] = 1; wf_failed[p->wf[k]] = 1;
            } else {
                phase[k] = WAIT_PRE;
            }
        }
        /* 3. decode admissions: the first waiting call of an instance, as long as it fits */
        for (uint32_t q = 0; q < p->Q; ++q) {
            for (;;) {
                int found = 0;
                uint32_t best = 0;
                for (uint32_t k = 0; k < K; ++k)
                    if (phase[k] == WAIT_DEC && dec_inst[k] == q && (!found || key[k] < key[best])) { best = k; found = 1; }
                if (!found) break;
                uint64_t need = (uint64_t)p->in_len[best] + p->out_len[best];
                if (used[q] + need > p->cap[q]) break;
                used[q] += need;
                phase[best] = IN_DEC;
                ds[best] = t;
                t_event[best] = t + decode_time(p, q, best);
            }
        }
        /* 4. prefill starts */
        for (uint32_t i = 0; i < p->P; ++i) {
            if (pre_busy[i]) continue;
            int found = 0;
            uint32_t best = 0;
            for (uint32_t k = 0; k < K; ++k)
                if (phase[k] == WAIT_PRE && pre_inst[k] == i && (!found || key[k] < key[best])) { best = k; found = 1; }
            if (!found) continue;
            pre_busy[i] = 1;
            phase[best] = IN_PRE;
            ps[best] = t;
            t_event[best] = t + prefill_time(p, i, best);
        }
    }

    /* workflows -> completion ratios -> metrics */
    ago_metrics m;
    memset(&m, 0, sizeof m);
    uint64_t first_arrival = W ? p->arrival_us[0] : 0, last_done = 0;
    for (uint32_t w = 0; w < W; ++w)
        if (p->arrival_us[w] < first_arrival) first_arrival = p->arrival_us[w];
    uint64_t *wf_done = calloc(W ? W : 1, 8);
    if (!wf_done) return 2;
    for (uint32_t w = 0; w < W; ++w) wf_done[w] = p->arrival_us[w];          /* a workflow without calls completes on arrival */
    for (uint32_t k = 0; k < K; ++k) {
        if (done[k] > wf_done[p->wf[k]]) wf_done[p->wf[k]] = done[k];
        if (done[k] > last_done) last_done = done[k];
    }
    for (uint32_t w = 0; w < W; ++w) {
        uint64_t c = wf_done[w] - p->arrival_us[w];
        ratio[w] = wf_failed[w] ? p->penalty_permille : c * 1000u / p->slo_us[w];
        m.sum_ratio_permille += ratio[w];
        if (wf_failed[w] || c > p->slo_us[w]) m.n_late++;
        if (wf_failed[w]) m.n_failed++;
    }
    m.makespan_us = last_done > first_arrival ? last_done - first_arrival : 0;
    if (W) {
        qsort(ratio, W, 8, cmp_u64);
        m.p95_permille = ratio[(95ull * W + 99u) / 100u - 1u];
        m.p99_permille = ratio[(99ull * W + 99u) / 100u - 1u];
    }
    *out = m;
    if (det) {
        for (uint32_t k = 0; k < K; ++k) {
            if (det->release_us) det->release_us[k] = rel[k];
            if (det->pre_start_us) det->pre_start_us[k] = ps[k];
            if (det->pre_end_us) det->pre_end_us[k] = pe[k];
            if (det->dec_start_us) det->dec_start_us[k] = ds[k];
            if (det->done_us) det->done_us[k] = done[k];
            if (det->failed) det->failed[k] = failed[k];
        }
    }
    free(phase); free(failed); free(wf_failed); free(pre_busy); free(t_event); free(done); free(used);
    free(rel); free(ps); free(pe); free(ds); free(ratio); free(wf_done);
    return 0;
}

int ago_eval_batch(const ago_problem *p, const uint16_t *pre_inst, const uint16_t *dec_inst, const uint32_t *key,
                   uint32_t C, ago_metrics *out)
{
    for (uint32_t c = 0; c < C; ++c) {
        int rc = ago_eval(p, pre_inst + (size_t)c * p->K, dec_inst + (size_t)c * p->K, key + (size_t)c * p->K, &out[c], NULL);
        if (rc) return rc;
    }
    return 0;
}
