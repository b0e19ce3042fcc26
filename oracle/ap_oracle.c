/*
 * CPU oracle for batched scoring of candidate request-to-replica assignments.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what the
 * GPU library must compute.  Only the tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it; the product never does.  It shares no code, header,
 * table or constant generator with the HIP path.
 *
 * What is computed, and which passage of the paper each step follows
 * ------------------------------------------------------------------
 *  - Every candidate is scored independently against the same snapshotted trace
 *    (Section 5.3 "Evaluator": the observed runtime trace is replayed against each
 *    candidate; Section 7.3 "Convergence analysis": candidates are evaluated
 *    independently).
 *  - A candidate is the workload-assignment dimension of a serving plan
 *    (Section 2.1 "Serving plans", item (i)): row[r] names the replica of request r.
 *    Within a replica requests are served in arrival order (the per-instance queue
 *    order of Section 8.3 "Agentic Request Scheduling", Setup); ties in arrival
 *    time are broken by request index.
 *  - A replica serves at most B requests at once: continuous batching with maximum
 *    per-replica batch size b^max (Section 5.3 "Serving simulator"; Notations table,
 *    b^max).  A request joins as soon as one of the B slots is free.
 *  - A request's service time is a prefill term plus a decode term that grows with
 *    its context (Appendix "Serving Simulator", serve-latency equation
 *    Lambda = T_prefill(s^p) + sum_k T_decode(k)).  The paper's roofline terms are
 *    replaced by an integer-microsecond linearisation:
 *        prefill = a + b * prompt_len
 *        tpot    = c + d * ceil(prompt_len / 1024)
 *        decode  = out_len * tpot
 *    with per-replica coefficients (a, b, c, d).
 *  - Replicas come and go (Section 4, data plane: the snapshot holds request arrival
 *    patterns and cluster resource availability; Section 8.2 "Elastic Cluster
 *    Dynamics").  Replica m exists during [t_on, t_off): nothing starts before t_on;
 *    a request whose start would be >= t_off is not served.  Requests already started
 *    run to completion (the drain of Appendix "Serving Simulator", reconfiguration
 *    cost).
 *  - A request that cannot be served (replica id >= M, or start >= t_off) is charged
 *    a large finite penalty latency instead of being dropped from the objective
 *    (Appendix "Serving Simulator", Memory Feasibility: infeasible choices get a
 *    penalty latency Lambda_inf >> 0).
 *  - The objective is per-request: latency is tracked per request through the replay
 *    and reduced to a percentile and to the number of requests meeting a latency
 *    threshold (Appendix "Discussion and Limitation", adaptability to diverse serving
 *    objectives), plus the trace completion time (Section 5.1 "Objective").
 *
 * Readings where the paper is silent (all stated again in the design notes):
 *  batch occupancy does not change a request's service time; all slots start free at
 *  time 0; the earliest-free slot is taken, lowest index on ties; TPOT is decode time
 *  per output token, which is exactly c + d*ceil(prompt/1024); SLO is met at equality;
 *  a rejected request counts with ttft = tpot = e2e = penalty in sums and histograms,
 *  never meets the SLO and never enters the makespan; percentiles use the nearest-rank rule over all R
 *  requests on a 4096-bin log-linear histogram and report the bin's lower edge.
 *
 * Pins (tests that run without a GPU): hand-worked traces, the single-slot Lindley
 * closed form, the order-statistic definition of the B-slot queue, sweep-line
 * invariants, brute force over all assignments of tiny instances, numpy reductions
 * for the no-wait case; the child-row rule against numpy's indexed assignment (last
 * write wins) and hand-made lists.  Nothing in this file is "parity unpinned".
 *
 * All times are unsigned 64-bit microseconds.
 */
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_BINS 4096u

typedef struct {
    uint32_t prefill_base_us;     /* a */
    uint32_t prefill_per_tok_us;  /* b */
    uint32_t decode_base_us;      /* c */
    uint32_t decode_per_kctx_us;  /* d, per started 1024 prompt tokens */
    uint64_t t_on_us;
    uint64_t t_off_us;
} orc_replica;

typedef struct {
    uint64_t sum_e2e_us;
    uint64_t sum_ttft_us;
    uint64_t sum_tpot_us;
    uint64_t makespan_us;
    uint64_t p99_ttft_us;
    uint64_t p99_tpot_us;
    uint64_t p99_e2e_us;
    uint32_t slo_ok;
    uint32_t n_rejected;
} orc_metrics;

typedef struct {
    uint32_t R;
    const uint64_t *arrival_us;
    const int32_t *prompt_len;
    const int32_t *out_len;
    uint32_t M;
    const orc_replica *replicas;
    uint32_t B;
    uint64_t slo_ttft_us;
    uint64_t slo_tpot_us;
    uint64_t penalty_us;
    /* Tabulated cost model (optional; all three NULL = the linear stand-in above).  The serving
     * simulator's estimate of a request's prefill time and of its time per output token on a
     * given kind of replica can come from any model - the paper's own is the roofline sum of
     * Appendix "Serving Simulator" - so here it is an input: replica m is of type rep_type[m]
     * (< n_types) and request r costs prefill_tab[type * R + r] microseconds of prefill and
     * tpot_tab[type * R + r] microseconds per output token there; decode = out_len * tpot as
     * before.  The coefficients of `replicas` are then unused; the windows still apply. */
    uint32_t n_types;
    const uint32_t *rep_type;
    const uint32_t *prefill_tab;
    const uint32_t *tpot_tab;
} orc_problem;

/* Optional per-request record of one replay, for the invariant tests. */
typedef struct {
    uint64_t *start_us;   /* [R]; undefined for rejected requests */
    uint64_t *finish_us;  /* [R] */
    uint64_t *ttft_us;    /* [R] */
    uint64_t *tpot_us;    /* [R] */
    uint64_t *e2e_us;     /* [R] */
    uint8_t *rejected;    /* [R] */
} orc_detail;

/* 4096-bin histogram: bins 0..127 hold the values 0..127 exactly; above that every
 * octave [2^e, 2^(e+1)) is cut into 128 equal sub-bins; everything from 2^38 - 2^30 up
 * falls in the last bin. */
uint32_t orc_hist_bin(uint64_t v)
{
    if (v < 128u) return (uint32_t)v;
    int e = 63 - __builtin_clzll(v);          /* floor(log2 v), >= 7 */
    if (e > 37) return ORC_BINS - 1u;
    uint32_t sub = (uint32_t)((v >> (e - 7)) & 127u);
    return ((uint32_t)(e - 6) << 7) | sub;
}

uint64_t orc_hist_lower(uint32_t bin)
{
    if (bin < 128u) return bin;
    uint32_t oct = bin >> 7;                  /* = e - 6 */
    return (uint64_t)(128u | (bin & 127u)) << (oct - 1u);
}

/* nearest-rank percentile: smallest bin whose cumulative count reaches k */
static uint64_t percentile_edge(const uint32_t *hist, uint64_t k)
{
    uint64_t cum = 0;
    for (uint32_t b = 0; b < ORC_BINS; ++b) {
        cum += hist[b];
        if (cum >= k) return orc_hist_lower(b);
    }
    return orc_hist_lower(ORC_BINS - 1u);
}

int orc_eval_row(const orc_problem *p, const uint16_t *row, orc_metrics *out, const orc_detail *det)
{
    const uint32_t R = p->R, M = p->M, B = p->B;
    if (R == 0 || M == 0 || B == 0) return 1;

    uint64_t *ttft = malloc(sizeof(uint64_t) * R);
    uint64_t *tpot = malloc(sizeof(uint64_t) * R);
    uint64_t *e2e = malloc(sizeof(uint64_t) * R);
    uint64_t *fin = malloc(sizeof(uint64_t) * R);
    uint64_t *sta = malloc(sizeof(uint64_t) * R);
    uint8_t *rej = malloc(R);
    uint32_t *queue = malloc(sizeof(uint32_t) * R);
    uint64_t *slot_free = malloc(sizeof(uint64_t) * B);
    uint32_t *hist = malloc(sizeof(uint32_t) * ORC_BINS * 3);
    if (!ttft || !tpot || !e2e || !fin || !sta || !rej || !queue || !slot_free || !hist) {
        free(ttft); free(tpot); free(e2e); free(fin); free(sta); free(rej); free(queue);
        free(slot_free); free(hist);
        return 2;
    }

    /* requests naming a replica that does not exist are rejected */
    for (uint32_t r = 0; r < R; ++r) {
        rej[r] = (row[r] >= M);
        sta[r] = 0; fin[r] = 0;
    }

    for (uint32_t m = 0; m < M; ++m) {
        const orc_replica *rep = &p->replicas[m];
        /* step 1: the replica's queue, in arrival (= index) order */
        uint32_t n = 0;
        for (uint32_t r = 0; r < R; ++r)
            if (row[r] == m) queue[n++] = r;

        /* step 2: B-slot first-come-first-served replay */
        for (uint32_t s = 0; s < B; ++s) slot_free[s] = 0;
        for (uint32_t i = 0; i < n; ++i) {
            uint32_t r = queue[i];
            uint64_t prompt = (uint64_t)p->prompt_len[r];
            uint64_t prefill = (uint64_t)rep->prefill_base_us + (uint64_t)rep->prefill_per_tok_us * prompt;
            uint64_t kctx = (prompt + 1023u) / 1024u;
            uint64_t per_tok = (uint64_t)rep->decode_base_us + (uint64_t)rep->decode_per_kctx_us * kctx;
            if (p->prefill_tab) {                   /* tabulated cost model */
                size_t at = (size_t)p->rep_type[m] * R + r;
                prefill = p->prefill_tab[at];
                per_tok = p->tpot_tab[at];
            }
            uint64_t decode = (uint64_t)p->out_len[r] * per_tok;

            uint32_t best = 0;
            for (uint32_t s = 1; s < B; ++s)
                if (slot_free[s] < slot_free[best]) best = s;

            uint64_t start = p->arrival_us[r];
            if (slot_free[best] > start) start = slot_free[best];
            if (rep->t_on_us > start) start = rep->t_on_us;

            if (start >= rep->t_off_us) {           /* replica gone: not served */
                rej[r] = 1;
                continue;
            }
            uint64_t finish = start + prefill + decode;
            slot_free[best] = finish;
            sta[r] = start;
            fin[r] = finish;
            ttft[r] = start - p->arrival_us[r] + prefill;
            tpot[r] = per_tok;
            e2e[r] = finish - p->arrival_us[r];
        }
    }

    /* steps 3-6: per-request values -> objectives */
    memset(hist, 0, sizeof(uint32_t) * ORC_BINS * 3);
    orc_metrics mt;
    memset(&mt, 0, sizeof mt);
    uint64_t last_finish = 0;
    int any_served = 0;
    for (uint32_t r = 0; r < R; ++r) {
        if (rej[r]) {
            ttft[r] = tpot[r] = e2e[r] = p->penalty_us;
            mt.n_rejected++;
        } else {
            if (!any_served || fin[r] > last_finish) last_finish = fin[r];
            any_served = 1;
        }
        /* an unserved request never meets the SLO, whatever the penalty value */
        if (!rej[r] && ttft[r] <= p->slo_ttft_us && tpot[r] <= p->slo_tpot_us) mt.slo_ok++;
        mt.sum_e2e_us += e2e[r];
        mt.sum_ttft_us += ttft[r];
        mt.sum_tpot_us += tpot[r];
        hist[orc_hist_bin(ttft[r])]++;
        hist[ORC_BINS + orc_hist_bin(tpot[r])]++;
        hist[2 * ORC_BINS + orc_hist_bin(e2e[r])]++;
    }
    mt.makespan_us = any_served ? last_finish - p->arrival_us[0] : 0;
    uint64_t k = (99ull * R + 99ull) / 100ull;     /* ceil(0.99 R) */
    mt.p99_ttft_us = percentile_edge(hist, k);
    mt.p99_tpot_us = percentile_edge(hist + ORC_BINS, k);
    mt.p99_e2e_us = percentile_edge(hist + 2 * ORC_BINS, k);
    *out = mt;

    if (det) {
        for (uint32_t r = 0; r < R; ++r) {
            if (det->start_us) det->start_us[r] = sta[r];
            if (det->finish_us) det->finish_us[r] = fin[r];
            if (det->ttft_us) det->ttft_us[r] = ttft[r];
            if (det->tpot_us) det->tpot_us[r] = tpot[r];
            if (det->e2e_us) det->e2e_us[r] = e2e[r];
            if (det->rejected) det->rejected[r] = rej[r];
        }
    }
    free(ttft); free(tpot); free(e2e); free(fin); free(sta); free(rej); free(queue);
    free(slot_free); free(hist);
    return 0;
}

/* ---- sparse candidates: a parent assignment plus per-child edit lists ------------
 * A child candidate is a small modification of a parent (Section 5.4 "Synthesis
 * Configuration", trade-off-aware mutation: children are diff-based modifications of a
 * high-performing parent; Section 6.1 "Warm-start re-evolution": a population holds top
 * candidates along with their mutations).  For the workload-assignment dimension the
 * diff is a list of (request, replica) pairs.  The child's row is the parent's row with
 * the list applied front to back: a later edit of the same request replaces an earlier
 * one, and an edit that names a request outside the trace changes nothing.  A replica id
 * outside the table is kept as it is (the replay rejects that request, as for any row).
 * The child's metrics are those of orc_eval_row on this row: nothing else is defined. */
void orc_child_row(const uint16_t *parent, uint32_t R, const uint32_t *request, const uint16_t *replica,
                   uint64_t n_edits, uint16_t *row)
{
    for (uint32_t r = 0; r < R; ++r) row[r] = parent[r];
    for (uint64_t e = 0; e < n_edits; ++e)
        if (request[e] < R) row[request[e]] = replica[e];
}

/* ---- many rows: threads over candidate rows, nothing else --------------------- */
typedef struct {
    const orc_problem *p;
    const uint16_t *assign;
    orc_metrics *out;
    uint32_t lo, hi;
    int rc;
} orc_job;

static void *orc_worker(void *arg)
{
    orc_job *j = arg;
    for (uint32_t c = j->lo; c < j->hi; ++c) {
        int rc = orc_eval_row(j->p, j->assign + (size_t)c * j->p->R, &j->out[c], NULL);
        if (rc) { j->rc = rc; break; }
    }
    return NULL;
}

int orc_eval_batch(const orc_problem *p, const uint16_t *assign, uint32_t C, uint32_t nthreads,
                   orc_metrics *out)
{
    if (nthreads == 0) nthreads = 1;
    if (nthreads > C) nthreads = C ? C : 1;
    pthread_t *tid = malloc(sizeof(pthread_t) * nthreads);
    orc_job *jobs = malloc(sizeof(orc_job) * nthreads);
    if (!tid || !jobs) { free(tid); free(jobs); return 2; }
    uint32_t per = (C + nthreads - 1) / nthreads;
    for (uint32_t t = 0; t < nthreads; ++t) {
        uint32_t lo = t * per, hi = lo + per;
        if (lo > C) lo = C;
        if (hi > C) hi = C;
        jobs[t] = (orc_job){p, assign, out, lo, hi, 0};
        pthread_create(&tid[t], NULL, orc_worker, &jobs[t]);
    }
    int rc = 0;
    for (uint32_t t = 0; t < nthreads; ++t) {
        pthread_join(tid[t], NULL);
        if (jobs[t].rc) rc = jobs[t].rc;
    }
    free(tid); free(jobs);
    return rc;
}
