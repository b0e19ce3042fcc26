/*
 * autopoiesis_eval.h -- C ABI of the MI355X (gfx950) candidate-assignment evaluator.
 *
 * The library scores many candidate request-to-replica assignments against one
 * observed request trace: the evaluator step of the paper's policy-evolution loop
 * (Section 5.3 "Evaluator": the snapshotted runtime trace is replayed against each
 * candidate; Section 7.3 "Convergence analysis": candidates are evaluated
 * independently), specialised to the workload-assignment dimension of a serving plan
 * (Section 2.1 "Serving plans", item (i)) and to per-request objectives (Appendix
 * "Discussion and Limitation", adaptability to diverse serving objectives: per-request
 * latency is tracked through the replay and reduced to a percentile or to the number
 * of requests meeting a latency threshold).
 *
 * Per candidate, requests are grouped by replica in arrival order, every replica is
 * replayed as a B-slot first-come-first-served continuous-batching queue (Section 5.3
 * "Serving simulator"; B is the maximum per-replica batch size b^max of the Notations
 * table) under an integer-microsecond prefill/decode cost model (the shape of the
 * serve-latency equation of Appendix "Serving Simulator": a prefill term plus a decode
 * term that grows with context), and the per-request latencies are reduced to the
 * ap_metrics record below.
 *
 * Around that call: candidates given as edit lists against a parent assignment
 * (ap_parent_set, ap_eval_children), cost models given as tables (ap_costtable_set) and the
 * paper's roofline cost model to fill them (ap_roofline_tables, ap_roofline_costs), the
 * end-to-end trace time of plan sequences with reconfiguration cost (ap_trace_time), and
 * candidate plans of multi-call agentic workflows (ap_agentic_*).  Each is documented at
 * its declaration with the passage of the paper it follows.
 *
 * All calls return an ap_status and never throw or abort.  Out-parameters are left
 * untouched on error.  Every kernel runs on the device that is current when the
 * workload is created; the evaluation is asynchronous on the caller's stream.
 */
#ifndef AUTOPOIESIS_EVAL_H
#define AUTOPOIESIS_EVAL_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ap_workload ap_workload; /* opaque; the library owns every device copy */

typedef enum {
    AP_OK = 0,
    AP_ERR_INVALID = 1, /* null pointer, zero size, unsorted arrivals, non-positive length ... */
    AP_ERR_RANGE = 2,   /* a documented capacity of the device path is exceeded */
    AP_ERR_ALLOC = 3,   /* host or device allocation failed */
    AP_ERR_DEVICE = 4,  /* a HIP call failed */
    AP_ERR_STATE = 5    /* evaluation requested before a cost model (for children: a parent) was set */
} ap_status;

/* One replica (Section 4, data plane: the snapshot carries cluster resource
 * availability; Section 8.2 "Elastic Cluster Dynamics").  Service time of a request on
 * this replica, in microseconds:
 *     prefill = prefill_base_us + prefill_per_tok_us * prompt_len
 *     tpot    = decode_base_us  + decode_per_kctx_us * ceil(prompt_len / 1024)
 *     decode  = out_len * tpot
 * The replica exists during [t_on_us, t_off_us): nothing starts before t_on_us; a
 * request whose start would be >= t_off_us is rejected; started requests drain.
 * Always available = {0, UINT64_MAX}. */
typedef struct {
    uint32_t prefill_base_us;
    uint32_t prefill_per_tok_us;
    uint32_t decode_base_us;
    uint32_t decode_per_kctx_us;
    uint64_t t_on_us;
    uint64_t t_off_us;
} ap_replica;

/* Latency thresholds (met at equality) and the latency charged to a request that is
 * not served (replica id >= M, or replica gone): the penalty latency of Appendix
 * "Serving Simulator", Memory Feasibility. */
typedef struct {
    uint64_t ttft_us;
    uint64_t tpot_us;
    uint64_t penalty_us;
} ap_slo;

/* Per-candidate result, 64 bytes.  Sums and counts run over all R requests; a rejected
 * request contributes ttft = tpot = e2e = penalty_us and never meets the SLO.
 * makespan_us = latest finish of a served request minus the first arrival (0 if none
 * was served): the trace completion time of Section 5.1 "Objective".
 * p99_* = nearest-rank 99th percentile (rank ceil(0.99 R)) on the 4096-bin histogram
 * of ap_hist_bin, reported as the lower edge of the bin. */
typedef struct {
    uint64_t sum_e2e_us;
    uint64_t sum_ttft_us;
    uint64_t sum_tpot_us;
    uint64_t makespan_us;
    uint64_t p99_ttft_us;
    uint64_t p99_tpot_us;
    uint64_t p99_e2e_us;
    uint32_t slo_ok;     /* requests with ttft <= slo.ttft_us and tpot <= slo.tpot_us */
    uint32_t n_rejected;
} ap_metrics;

/* Capacities of the device path (exceeding one gives AP_ERR_RANGE, never a wrong result). */
#define AP_MAX_SLOTS 64u      /* B */
#define AP_MAX_REPLICAS 1024u /* M */

/* Take a trace snapshot (Section 4: a sliding window of request arrivals).
 *   arrival_us, prompt_len, out_len : HOST arrays of R elements, copied; the caller keeps its buffers.
 *   arrival_us must be non-decreasing; prompt_len and out_len must be >= 1; R >= 1.
 * On success *out owns device copies on the current device.  Errors: AP_ERR_INVALID, AP_ERR_ALLOC,
 * AP_ERR_DEVICE. */
ap_status ap_workload_create(const uint64_t *arrival_us, const int32_t *prompt_len, const int32_t *out_len,
                             uint32_t R, ap_workload **out);

/* Attach (or replace) the replica table, the slot count and the SLOs.
 *   replicas : HOST array of M entries, copied.  1 <= M <= AP_MAX_REPLICAS, 1 <= B <= AP_MAX_SLOTS,
 *              t_on_us <= t_off_us for every replica (AP_ERR_INVALID otherwise).
 * The device keeps time as 32-bit microseconds relative to the first arrival.  The call
 * proves that no finish time can leave that range (latest arrival or t_on, plus the sum
 * of every request's largest service time, must be below 2^32 - 1 us, about 71 minutes);
 * otherwise it returns AP_ERR_RANGE and the workload keeps its previous cost model, if any.
 * It also decides which kernels later evaluations run and sizes every device buffer they need:
 * replicas that differ or have windows, crowded traces and very small tables are scored by an
 * evaluation that replays per-replica request lists, whose scratch area (lists for one batch of
 * candidates, at most 4 GiB) is allocated here; when M*B slot times of one candidate do not fit
 * in LDS next to the histograms, what is left for the general replay goes through a three-kernel
 * path with a scratch area of about 1 GiB, allocated here as well.  A device that cannot provide
 * the lists' area (or a trace so long that 64 candidates' lists exceed 8 GiB) only loses that
 * evaluation - the general replay scores the calls instead; AP_ERR_ALLOC if it cannot provide
 * the three-kernel path's area.
 * Synchronous (small host-to-device copies, one small kernel). */
ap_status ap_costmodel_set(ap_workload *w, const ap_replica *replicas, uint32_t M, uint32_t B, const ap_slo *slo);

/* A replica whose service times come from tables: its type selects the table row, its window
 * is as in ap_replica. */
typedef struct {
    uint32_t type;
    uint64_t t_on_us;
    uint64_t t_off_us;
} ap_typed_replica;

/* Attach (or replace) a tabulated cost model: the serving simulator's estimate of every request's
 * prefill time and time per output token on every kind of replica is an input, so any cost model
 * can be plugged in - the paper's own is the roofline sum of Appendix "Serving Simulator"
 * (serve-latency equation: T_prefill(s^p) plus the decode steps).  Service time of request r on a
 * replica of type t, in microseconds:
 *     prefill = prefill_us[t * R + r],   tpot = tpot_us[t * R + r],   decode = out_len[r] * tpot
 * Everything else (B slots, windows, SLOs, penalty, metrics) is as for ap_costmodel_set, and so are
 * the range proof (AP_ERR_RANGE, previous model kept), the sizing of device buffers and the errors.
 *   replicas            : HOST array of M entries, copied; type < n_types (AP_ERR_INVALID otherwise).
 *   prefill_us, tpot_us : HOST arrays, uint32 [n_types][R], copied.  n_types * R must be below 2^32.
 * Synchronous.  Replaces a model set by ap_costmodel_set and vice versa; discards the parent, if any. */
ap_status ap_costtable_set(ap_workload *w, const ap_typed_replica *replicas, uint32_t M, uint32_t B, const ap_slo *slo,
                           const uint32_t *prefill_us, const uint32_t *tpot_us, uint32_t n_types);

/* Score C candidates.
 *   d_assign : DEVICE pointer, uint16 [C][R] row-major; d_assign[c*R + r] is the replica of request r
 *              under candidate c.  A value >= M is not an error: that request is rejected.
 *   d_out    : DEVICE pointer to C ap_metrics records (8-byte aligned); only these are written.
 *   hip_stream : a hipStream_t passed as void* (NULL = the default stream).
 * Asynchronous: kernels are enqueued on hip_stream and the call returns without waiting.
 * It allocates nothing, copies nothing and clears nothing outside its kernels, so the call may be
 * captured into a HIP graph (stream capture on hip_stream) and replayed as long as the workload,
 * its cost model and both buffers stay as they were.  One evaluation per workload may be in
 * flight at a time.  C == 0 is a no-op.  Errors: AP_ERR_INVALID (null pointers), AP_ERR_STATE, AP_ERR_DEVICE.
 * The handle is const because the trace and the cost model are not changed, but the call does update host-side
 * bookkeeping inside it (which of two device flag words the call uses, the count of candidates scored): calls
 * on one workload, of this or any other kind, must come from one host thread at a time. */
ap_status ap_eval_candidates(const ap_workload *w, const uint16_t *d_assign, uint32_t C, ap_metrics *d_out,
                             void *hip_stream);

/* How the candidates scored since the last ap_costmodel_set / ap_costtable_set were settled: all of them, and
 * those among them that had to go through the request-by-request replay of every replica's queue (the others were
 * settled by one of the exact shortcuts: proven free of waiting, or split into a replayed backlog and a part that
 * starts on arrival).  A 32-bit device counter behind `replayed`: it wraps after 2^32 replayed candidates.
 * Synchronous: waits for the device.  Errors: AP_ERR_INVALID, AP_ERR_STATE, AP_ERR_DEVICE. */
typedef struct {
    uint64_t candidates;
    uint64_t replayed;
} ap_eval_counts;

ap_status ap_eval_counts_get(const ap_workload *w, ap_eval_counts *out);

/* Sparse candidates: children of one parent assignment (Section 5.4 "Synthesis Configuration",
 * trade-off-aware mutation: children are diff-based modifications of a high-performing parent;
 * Section 6.1 "Warm-start re-evolution": a population holds top candidates along with their
 * mutations).  For the workload-assignment dimension a child is the parent row plus a list of
 * (request, replica) edits.
 *
 * ap_parent_set fixes the parent for later ap_eval_children calls.
 *   parent       : HOST array, uint16 [R], copied.  Values >= M are allowed (those requests are rejected).
 *   max_children : the largest C a later ap_eval_children may pass (>= 1).  The call allocates
 *                  max_children * R * 2 bytes of device memory for the rows of children that need the
 *                  dense path (kept, and reused by later calls that ask for no more).
 * Needs a cost model (AP_ERR_STATE otherwise); a later ap_costmodel_set discards the parent.
 * Synchronous (one copy, one small kernel).  Errors: AP_ERR_INVALID, AP_ERR_STATE, AP_ERR_ALLOC, AP_ERR_DEVICE. */
ap_status ap_parent_set(ap_workload *w, const uint16_t *parent, uint32_t max_children);

/* Score C children of the parent.  Child c owns the edits e = d_edit_first[c] .. d_edit_first[c+1]-1
 * (none if that range is empty or reversed); its row is the parent's with
 * row[d_edit_request[e]] = d_edit_replica[e] applied in that order: a later edit of the same request
 * replaces an earlier one, an edit whose request is >= R changes nothing, a replica >= M is not an error
 * (that request is rejected).  d_out[c] is exactly what ap_eval_candidates returns for that row.
 *   d_edit_first   : DEVICE pointer, uint32 [C + 1].
 *   d_edit_request : DEVICE pointer, uint32 [E], E >= every index used by d_edit_first (must be a valid
 *   d_edit_replica : DEVICE pointer, uint16 [E]   pointer even when every list is empty).
 *   d_out          : DEVICE pointer to C ap_metrics records; only these are written.
 * Asynchronous on hip_stream, allocates nothing, launches kernels only (may be captured into a HIP
 * graph).  One evaluation per workload, of either kind, may be in flight at a time.  C == 0 is a no-op.
 * Errors: AP_ERR_INVALID (null pointers), AP_ERR_STATE (no cost model or no parent), AP_ERR_RANGE
 * (C > max_children), AP_ERR_DEVICE.  Like ap_eval_candidates the call updates host-side bookkeeping in the
 * handle: one host thread at a time per workload. */
ap_status ap_eval_children(const ap_workload *w, const uint32_t *d_edit_first, const uint32_t *d_edit_request,
                           const uint16_t *d_edit_replica, uint32_t C, ap_metrics *d_out, void *hip_stream);

/* Roofline cost tables (Appendix "Serving Simulator").  A model M_z is described by its layers L,
 * hidden size H, MLP intermediate size I, vocabulary V, attention heads A, key-value heads K <= A
 * and weight precision eta in bits (per-head dimension d = H / A); a GPU type g by its memory m_g
 * (bytes), peak throughput F_g (FLOP/s), HBM bandwidth B_g, PCIe bandwidth P_g, GPUs per node nu_g
 * and the interconnect bandwidth R inside a node and across nodes (all bytes/s); a replica group by
 * (z, g, tensor-parallel degree t, per-replica batch b). */
typedef struct {
    uint32_t layers, hidden, intermediate, vocab, heads, kv_heads, weight_bits;
} ap_model;

typedef struct {
    double mem_bytes, flops, hbm_bytes_per_s, pcie_bytes_per_s, link_intra_bytes_per_s, link_inter_bytes_per_s;
    uint32_t gpus_per_node;
} ap_gpu;

typedef struct {
    uint32_t model, gpu, tp, batch;
} ap_group;

/* Evaluate the serve-latency equation's two terms for every group and sequence length:
 *   prefill_ns[g][s], s = 0 .. max_seq       : T_prefill(z,g,t,b,s) in nanoseconds (entry 0 is 0);
 *   decode_prefix_ns[g][k], k = 0 .. max_seq+1 : sum of T_decode(z,g,t,b,j) over 1 <= j < k, so that the
 *       decode sum over k = s_p .. s_p + s_d - 1 is decode_prefix_ns[s_p + s_d] - decode_prefix_ns[s_p];
 *   weight_bytes[g] : W_z of the weight-size equation;  feasible[g] : 0 if W_z / t > 0.8 m_g, else 1.
 * Each term applies the roofline equations (pi = min(F / A * B_g, F_g), T = F / pi) to the QKV
 * projection, attention, output projection and MLP of a layer, L times, and to the output head once,
 * and adds the ring all-reduce time 2(t-1)/t * 2L * H * b * s * eta/8 / R_{g,t} (R: inside a node when
 * t <= nu_g).  Times are rounded to whole nanoseconds (half to even) before they are summed.
 * All pointers are HOST pointers; the four outputs must hold n_groups*(max_seq+1), n_groups*(max_seq+2),
 * n_groups and n_groups elements.  Synchronous; allocates and frees its own device buffers.
 * Errors: AP_ERR_INVALID (null pointers, empty arrays, an index out of range, a zero field, K > A, a
 * non-positive rate), AP_ERR_RANGE (more than 65535 groups, max_seq above 2^24), AP_ERR_ALLOC, AP_ERR_DEVICE. */
ap_status ap_roofline_tables(const ap_model *models, uint32_t n_models, const ap_gpu *gpus, uint32_t n_gpus,
                             const ap_group *groups, uint32_t n_groups, uint32_t max_seq, uint64_t *prefill_ns,
                             uint64_t *decode_prefix_ns, double *weight_bytes, uint8_t *feasible);

/* The same tables turned into the inputs of ap_costtable_set for the requests of a workload: for group g
 * (= replica type g) and request r with prompt length s_p and output length s_d,
 *   prefill_us[g * R + r] = (prefill_ns[g][s_p] + 500) / 1000
 *   tpot_us[g * R + r]    = (decode sum in ns + 500 s_d) / (1000 s_d)      (rounded time per output token)
 *   prefill_us, tpot_us : HOST pointers, uint32 [n_groups][R], written.
 * Synchronous.  Errors as above, AP_ERR_RANGE also when a request's s_p + s_d exceeds 2^24. */
ap_status ap_roofline_costs(const ap_workload *w, const ap_model *models, uint32_t n_models, const ap_gpu *gpus,
                            uint32_t n_gpus, const ap_group *groups, uint32_t n_groups, uint32_t *prefill_us,
                            uint32_t *tpot_us);

/* ap_roofline_costs and ap_costtable_set in one call, without the tables leaving the device: the roofline
 * terms of Appendix "Serving Simulator" (serve-latency equation) are evaluated for every group, turned into
 * prefill_us / tpot_us of every request of the workload exactly as ap_roofline_costs does, and written straight
 * into the workload's own table buffers; group g is replica type g (replicas[m].type < n_groups, AP_ERR_INVALID
 * otherwise).  The range proof of ap_costmodel_set runs as a reduction over the device tables, and the host
 * reads back its 32-byte result: no table is copied in either direction.  The roofline buffers and the table
 * buffers stay with the workload and are reused by later calls that fit (allocation only when they grow).
 *   replicas, models, gpus, groups : HOST arrays, copied.
 * Synchronous, like ap_costmodel_set (the host sizes LDS and scratch from the bounds).  Errors as for
 * ap_roofline_costs and ap_costtable_set; unlike those, a failure after the descriptions were validated leaves the
 * workload WITHOUT a cost model (the previous tables are overwritten before the proof can run). */
ap_status ap_costtable_set_roofline(ap_workload *w, const ap_typed_replica *replicas, uint32_t M, uint32_t B,
                                    const ap_slo *slo, const ap_model *models, uint32_t n_models, const ap_gpu *gpus,
                                    uint32_t n_gpus, const ap_group *groups, uint32_t n_groups);

/* End-to-end trace time of candidate plan sequences (Section 5.1, execution model):
 *   T_total = t_sched(1) + t_serve(1) + sum_{i=2}^{N} [ t_stale(i) + t_reconfig(i) + t_serve(i) ]
 * with t_reconfig(i) = Reconfig-Cost(sigma_{i-1}, sigma_i) = T_term + T_load of Appendix "Serving
 * Simulator", Reconfiguration Cost: tau(z, g) = W_z / P_g * c_z is the weight transfer time of model z on
 * GPU type g (W_z by the weight-size equation, c_z = pcie_coef[z]).  With Delta M the models whose (GPU
 * type, TP, count) tuples differ between the two plans, the termination-cost equation gives T_term = the
 * largest tau(z, g) over z in Delta M and the GPU types g the previous plan deploys z on, and the
 * loading-cost equation gives T_load(sigma_i) = the largest tau(z, g) over the GPU types g and EVERY model
 * z the new plan deploys on g, changed or not (AP_LOAD_DEPLOYED, the equation as printed).
 * AP_LOAD_CHANGED restricts the loading cost to z in Delta M as well - an alternative reading of "the time
 * to transfer new model weights", not the printed formula.  Equal plans (Delta M empty) cost nothing under
 * either.  The record is the evaluator's artifact feedback (Section 5.3, Table 1; the table's N counts
 * reschedulings, n_intervals here counts intervals including the cold start). */
#define AP_LOAD_DEPLOYED 0u
#define AP_LOAD_CHANGED 1u

typedef struct {
    uint32_t tp;    /* tensor-parallel degree of the model's replicas on this GPU type */
    uint32_t count; /* number of replicas; 0 = the model is not deployed on this GPU type */
} ap_placement;

typedef struct {
    uint64_t total_ns;
    uint64_t sum_stale_ns;
    uint64_t sum_reconfig_ns;
    uint64_t sum_serve_ns;
    uint64_t sched_ns;
    uint32_t n_intervals;
    uint32_t reserved;
} ap_breakdown;

/*   models, pcie_coef, gpus : HOST arrays (n_models, n_models, n_gpus entries); of ap_gpu only
 *                             pcie_bytes_per_s is used.
 *   d_plans       : DEVICE, ap_placement [C][N_max][n_models][n_gpus]; plan i of candidate c is sigma_{i+1}.
 *   d_n_intervals : DEVICE, uint32 [C]; N of each candidate, taken as at least 1 and at most N_max.
 *   d_sched_ns    : DEVICE, uint64 [C]; t_sched(1).
 *   d_stale_ns, d_serve_ns : DEVICE, uint64 [C][N_max]; t_stale(i+1), t_serve(i+1) at index i (stale[0] unused).
 *   load_scope    : AP_LOAD_DEPLOYED or AP_LOAD_CHANGED (above).
 *   d_out         : DEVICE, ap_breakdown [C], written.
 *   hip_stream    : a hipStream_t passed as void* (NULL = the default stream).  The kernels run on it, i.e.
 *                   behind whatever produced the device inputs there (e.g. serve times taken from an
 *                   ap_eval_candidates call on the same stream).
 * All times are nanoseconds.  The call allocates small temporary device buffers and frees them before it
 * returns, so it waits for hip_stream: d_out is complete on return.  C == 0 is a no-op.
 * Errors: AP_ERR_INVALID (null pointers, empty arrays, a zero model field, a non-positive coefficient or
 * bandwidth, an unknown load_scope), AP_ERR_RANGE (n_models * n_gpus above 2^20), AP_ERR_ALLOC, AP_ERR_DEVICE. */
ap_status ap_trace_time(const ap_model *models, const double *pcie_coef, uint32_t n_models, const ap_gpu *gpus,
                        uint32_t n_gpus, const ap_placement *d_plans, const uint32_t *d_n_intervals,
                        const uint64_t *d_sched_ns, const uint64_t *d_stale_ns, const uint64_t *d_serve_ns, uint32_t C,
                        uint32_t N_max, uint32_t load_scope, ap_breakdown *d_out, void *hip_stream);

/* ap_trace_time for callers that cannot allocate device memory or wait: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same results as ap_trace_time, but the
 * transfer-time table tau(z, g) is kept in a fixed array inside the library (8 KiB of device memory per GPU the
 * library runs on, held until the process ends) and the model / GPU descriptions travel in the kernel arguments,
 * so the call allocates nothing, frees nothing, copies nothing and does not wait: two kernels are queued on
 * hip_stream and d_out is complete when the stream reaches the end of them.
 * Limits: n_models <= AP_STATIC_MAX_MODELS, n_gpus <= AP_STATIC_MAX_GPU_TYPES, else AP_ERR_RANGE.
 * Every call on a GPU uses that GPU's one array: calls that overlap in time on one GPU (different streams, or
 * different host threads) race on it and must be serialised by the caller; calls on one stream are in order.
 * The array keeps the last call's table; each call rewrites every entry it reads.
 * Errors otherwise as ap_trace_time (AP_ERR_ALLOC cannot occur). */
#define AP_STATIC_MAX_MODELS 64u
#define AP_STATIC_MAX_GPU_TYPES 16u
ap_status ap_trace_time_static(const ap_model *models, const double *pcie_coef, uint32_t n_models, const ap_gpu *gpus,
                               uint32_t n_gpus, const ap_placement *d_plans, const uint32_t *d_n_intervals,
                               const uint64_t *d_sched_ns, const uint64_t *d_stale_ns, const uint64_t *d_serve_ns,
                               uint32_t C, uint32_t N_max, uint32_t load_scope, ap_breakdown *d_out, void *hip_stream);

/* Agentic request scheduling (Section 8.3; Appendix "Scheduling Problem Formulation", Formulation for
 * Agentic Request): multi-call workflows on a disaggregated cluster of prefill instances (one call at a
 * time) and decode instances (each with a token-capacity budget).  A call becomes schedulable when its
 * workflow has arrived and all its predecessor calls have completed.  A candidate plan gives every call
 * a prefill instance, a decode instance and a queue key; on every instance the waiting call with the
 * smallest (key, call index) goes first, a decode instance admitting its first waiting call as soon as
 * in_len + out_len tokens fit the free part of its budget (no overtaking).  Events of one instant are
 * applied as decode completions, prefill completions, releases, decode admissions, prefill starts.
 * Prefill of call k on instance p takes base_us + per_tok_us * in_len[k]; decode on instance q takes
 * out_len[k] * (base_us + per_kctx_us * ceil(in_len[k] / 1024)).  A call naming no prefill instance
 * fails at its release; one naming no decode instance, or larger than that instance's whole budget,
 * fails when its prefill ends; a failed call counts as completed then, and its workflow is charged
 * penalty_permille.  Per workflow: ratio = completion time * 1000 / SLO (the completion ratio C / SLO in
 * per mille). */
typedef struct ap_agentic ap_agentic;

typedef struct {
    uint32_t base_us, per_tok_us;
} ap_prefill_instance;

typedef struct {
    uint32_t base_us, per_kctx_us, capacity_tokens;
} ap_decode_instance;

/* Per candidate, 40 bytes: sum of the W ratios (mean = sum / W), their nearest-rank 95th and 99th
 * percentiles (rank ceil(q W / 100)), latest completion minus earliest arrival, workflows with C > SLO
 * (failed ones included), workflows with a failed call. */
typedef struct {
    uint64_t sum_ratio_permille;
    uint64_t p95_permille;
    uint64_t p99_permille;
    uint64_t makespan_us;
    uint32_t n_late;
    uint32_t n_failed;
} ap_agentic_metrics;

#define AP_AGENTIC_MAX_CALLS 1024u
#define AP_AGENTIC_MAX_WORKFLOWS 1024u
#define AP_AGENTIC_MAX_INSTANCES 64u /* of either kind */

/* All arrays are HOST arrays, copied.
 *   arrival_us, slo_us : [W]; slo_us > 0.
 *   wf, in_len, out_len : [K]; wf[k] < W; lengths >= 1.
 *   pred_first [K + 1], pred : predecessors of call k are pred[pred_first[k] .. pred_first[k+1]); each must be
 *       smaller than k and belong to the same workflow.
 *   prefill [P], decode [Q] : base_us + per_tok_us >= 1 resp. base_us + per_kctx_us >= 1 (no stage takes no time).
 * Errors: AP_ERR_INVALID (any of the above violated, null pointers, W, K, P or Q zero), AP_ERR_RANGE (a
 * capacity above exceeded, or arrivals plus all stage times could leave 32-bit microseconds), AP_ERR_ALLOC,
 * AP_ERR_DEVICE. */
ap_status ap_agentic_create(const uint64_t *arrival_us, const uint64_t *slo_us, uint32_t W, const uint32_t *wf,
                            const uint32_t *in_len, const uint32_t *out_len, const uint32_t *pred_first,
                            const uint32_t *pred, uint32_t K, const ap_prefill_instance *prefill, uint32_t P,
                            const ap_decode_instance *decode, uint32_t Q, uint64_t penalty_permille, ap_agentic **out);

/* Score C candidate plans.
 *   d_prefill, d_decode : DEVICE, uint16 [C][K]; an id >= P resp. >= Q is not an error (the call fails).
 *   d_key               : DEVICE, uint32 [C][K].
 *   d_out               : DEVICE, ap_agentic_metrics [C], written.
 * Asynchronous on hip_stream; allocates nothing; one kernel.  C == 0 is a no-op.
 * Errors: AP_ERR_INVALID (null pointers), AP_ERR_DEVICE. */
ap_status ap_agentic_eval(const ap_agentic *a, const uint16_t *d_prefill, const uint16_t *d_decode, const uint32_t *d_key,
                          uint32_t C, ap_agentic_metrics *d_out, void *hip_stream);

ap_status ap_agentic_destroy(ap_agentic *a);

/* Release the workload and its device memory.  NULL is accepted. */
ap_status ap_workload_destroy(ap_workload *w);

const char *ap_status_str(ap_status s);

/* The histogram behind the p99 fields (host helpers; the device uses the same map).
 * Bins 0..127 hold 0..127 exactly; each octave [2^e, 2^(e+1)), e >= 7, is cut into 128
 * equal sub-bins; values >= 2^38 - 2^30 us fall in bin 4095. */
uint32_t ap_hist_bin(uint64_t value_us);
uint64_t ap_hist_lower(uint32_t bin);

#ifdef __cplusplus
}
#endif
#endif /* AUTOPOIESIS_EVAL_H */
