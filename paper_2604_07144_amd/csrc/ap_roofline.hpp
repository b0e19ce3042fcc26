// Roofline cost tables: prefill time and decode-step time of every (model, GPU type, tensor-parallel degree,
// batch) group for every sequence length, and from them the per-request table entries of the tabulated cost
// model.
#ifndef AP_ROOFLINE_HPP
#define AP_ROOFLINE_HPP

#include "ap_common.hpp"

namespace {

// ----------------------------------------------------------------------------------
// the cost model of Appendix "Serving Simulator", in double precision
// ----------------------------------------------------------------------------------
// One group (z, g, t, b) of the serve-latency equation with everything the sublayer formulas
// need, as doubles.
struct RoofGroup {
    double L, H, I, V, A, K;      // layers, hidden, MLP intermediate, vocabulary, heads, key-value heads
    double e;                     // bytes per weight (eta / 8)
    double b, t;                  // batch, tensor-parallel degree
    double flops, hbm;            // F_g, B_g
    double link;                  // R_{g,t}: intra-node when t <= nu_g, cross-node otherwise
    double mem;                   // m_g
};

// Model weight size: W_z = [L (3 H I + 2 A H d + 2 K H d) + 2 H V] * eta / 8.
__device__ __forceinline__ double roof_weight_bytes(const RoofGroup& g) {
#pragma clang fp contract(off)
    const double d = g.H / g.A;
    const double per_layer = ((((3.0 * g.H) * g.I) + (((2.0 * g.A) * g.H) * d)) + (((2.0 * g.K) * g.H) * d));
    return ((g.L * per_layer) + ((2.0 * g.H) * g.V)) * g.e;
}

// Roofline equations: achieved performance pi = min(F / A * B_g, F_g), time F / pi.
__device__ __forceinline__ double roof_op_time(double flops, double bytes, const RoofGroup& g) {
#pragma clang fp contract(off)
    const double perf = fmin((flops / bytes) * g.hbm, g.flops);
    return flops / perf;
}

// One forward pass of n new tokens per sequence over a context of c tokens: the four sublayers of a
// layer (QKV projection, attention, output projection, MLP) L times, the output head once, and the two
// ring all-reduces per layer of the all-reduce equation.  Operations are written in one fixed order, with
// no fused multiply-add, so that the same arithmetic in any IEEE double implementation gives the same bits.
__device__ __forceinline__ double roof_phase_time(const RoofGroup& g, double n, double c) {
#pragma clang fp contract(off)
    const double d = g.H / g.A;
    const double qkv_w = g.A + 2.0 * g.K;
    const double qkv = roof_op_time(((((((2.0 * g.b) * n) * g.H) * qkv_w) * d) / g.t),
                                    g.e * (((((g.H * qkv_w) * d) / g.t) + ((g.b * n) * g.H)) + ((((g.b * n) * qkv_w) * d) / g.t)), g);
    const double att = roof_op_time(((((((4.0 * g.b) * n) * c) * g.A) * d) / g.t),
                                    g.e * ((((((2.0 * g.b) * n) * g.A) * d) / g.t) + (((((2.0 * g.b) * c) * g.K) * d) / g.t)), g);
    const double proj = roof_op_time(((((((2.0 * g.b) * n) * g.A) * d) * g.H) / g.t),
                                     g.e * (((((g.A * d) * g.H) / g.t) + ((((g.b * n) * g.A) * d) / g.t)) + ((g.b * n) * g.H)), g);
    const double mlp = roof_op_time((((((6.0 * g.b) * n) * g.H) * g.I) / g.t),
                                    g.e * (((((3.0 * g.H) * g.I) / g.t) + (((2.0 * g.b) * n) * g.H)) + ((((3.0 * g.b) * n) * g.I) / g.t)), g);
    const double head = roof_op_time(((((2.0 * g.b) * g.H) * g.V) / g.t),
                                     g.e * ((((g.H * g.V) / g.t) + (g.b * g.H)) + ((g.b * g.V) / g.t)), g);
    double comm = 0.0;
    if (g.t != 1.0) comm = (((((((2.0 * (g.t - 1.0)) / g.t) * (2.0 * g.L)) * g.H) * g.b) * n) * g.e) / g.link;
    return ((g.L * (((qkv + att) + proj) + mlp)) + head) + comm;
}

__device__ __forceinline__ unsigned long long roof_ns(double seconds) {
#pragma clang fp contract(off)
    return (unsigned long long)__double2ll_rn(seconds * 1e9);              // round half to even
}

constexpr uint32_t kRoofThreads = 256;

// prefill_ns[g][s] for s = 0 .. max_seq (entry 0 is 0) and step_ns[g][k], the decode step at context
// k (entry 0 is 0: a context holds at least one token).  One thread per (group, length).
// Also, once per group: its weight size and the memory-feasibility verdict W_z / t <= 0.8 m_g.
__global__ __launch_bounds__(kRoofThreads) void k_roofline_steps(const RoofGroup* __restrict__ groups, uint32_t n_groups,
                                                                 uint32_t max_seq, unsigned long long* __restrict__ prefill_ns,
                                                                 unsigned long long* __restrict__ step_ns,
                                                                 double* __restrict__ weight_bytes,
                                                                 uint32_t* __restrict__ feasible) {
    const uint32_t s = blockIdx.x * kRoofThreads + threadIdx.x, gi = blockIdx.y;
    if (s > max_seq || gi >= n_groups) return;
    const RoofGroup g = groups[gi];
    if (s == 0u) {
        const double w = roof_weight_bytes(g);
        weight_bytes[gi] = w;
        feasible[gi] = (w / g.t > 0.8 * g.mem) ? 0u : 1u;
    }
    const size_t at = (size_t)gi * (max_seq + 1u) + s;
    prefill_ns[at] = s == 0u ? 0ull : roof_ns(roof_phase_time(g, (double)s, (double)s));
    step_ns[at] = s == 0u ? 0ull : roof_ns(roof_phase_time(g, 1.0, (double)s));
}

// prefix_ns[g][k] = sum of step_ns[g][j] for j < k, k = 0 .. max_seq + 1: the sum of the serve-latency
// equation over k = s_p .. s_p + s_d - 1 is then prefix[s_p + s_d] - prefix[s_p].  Integers: the order of
// the additions does not matter.  One workgroup per group walks its row in tiles.
__global__ __launch_bounds__(kRoofThreads) void k_roofline_prefix(const unsigned long long* __restrict__ step_ns,
                                                                  uint32_t max_seq, unsigned long long* __restrict__ prefix_ns) {
    __shared__ unsigned long long wave_total[kRoofThreads / kWave];
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wv = tid >> 6, gi = blockIdx.x;
    const unsigned long long* in = step_ns + (size_t)gi * (max_seq + 1u);
    unsigned long long* out = prefix_ns + (size_t)gi * (max_seq + 2u);
    unsigned long long carry = 0ull;
    if (tid == 0u) out[0] = 0ull;
    for (uint32_t base = 0; base <= max_seq; base += kRoofThreads) {
        const uint32_t k = base + tid;
        unsigned long long v = k <= max_seq ? in[k] : 0ull;
#pragma unroll
        for (uint32_t dlt = 1; dlt < kWave; dlt <<= 1) {
            const unsigned long long up = (unsigned long long)__shfl_up((long long)v, dlt);
            if (lane >= dlt) v += up;
        }
        if (lane == 63u) wave_total[wv] = v;
        __syncthreads();
        unsigned long long before = carry, total = carry;
#pragma unroll
        for (uint32_t j = 0; j < kRoofThreads / kWave; ++j) {
            before += j < wv ? wave_total[j] : 0ull;
            total += wave_total[j];
        }
        if (k <= max_seq) out[k + 1u] = before + v;                            // inclusive sum up to k = prefix of k + 1
        carry = total;
        __syncthreads();
    }
}

// Table entries of the tabulated cost model for a trace: per group and request,
// prefill_us = T_prefill(s_p) rounded to microseconds, tpot_us = the decode sum of the serve-latency
// equation divided by the number of output tokens, rounded.
__global__ __launch_bounds__(kRoofThreads) void k_roofline_request_costs(const unsigned long long* __restrict__ prefill_ns,
                                                                         const unsigned long long* __restrict__ prefix_ns,
                                                                         uint32_t max_seq, const uint32_t* __restrict__ prompt,
                                                                         const uint32_t* __restrict__ outlen, uint32_t R,
                                                                         uint32_t* __restrict__ prefill_us,
                                                                         uint32_t* __restrict__ tpot_us) {
    const uint32_t r = blockIdx.x * kRoofThreads + threadIdx.x, gi = blockIdx.y;
    if (r >= R) return;
    const uint32_t sp = prompt[r], sd = outlen[r];                            // the host checked sp + sd <= max_seq
    const unsigned long long pre = prefill_ns[(size_t)gi * (max_seq + 1u) + sp];
    const unsigned long long* prefix = prefix_ns + (size_t)gi * (max_seq + 2u);
    const unsigned long long decode = prefix[sp + sd] - prefix[sp];
    const unsigned long long pre_us = (pre + 500ull) / 1000ull;
    const unsigned long long per_tok = (decode + 500ull * sd) / (1000ull * sd);
    prefill_us[(size_t)gi * R + r] = (uint32_t)min(pre_us, 0xFFFFFFFFull);
    tpot_us[(size_t)gi * R + r] = (uint32_t)min(per_tok, 0xFFFFFFFFull);
}

// What the host has to know about cost tables that never leave the device before it accepts them: with the
// service time of request r taken as its longest over the replica types in use (prefill + out_len * tpot),
//   service_sum     all of them added up (each clamped to 2^33, far beyond what 32-bit time allows anyway),
//   latest_unqueued the latest arrival + service time,
//   longest_pair    the longest time from the arrival of request 2q to the unqueued finish of 2q or 2q + 1,
//   over_range      how many table entries reach the value reserved for "never",
//   longest_prefill, longest_tpot   the largest entries of the rows in use;
// and per request its longest service time (clamped to 32 bits), for the host's sweep over the trace.
struct TableBounds {
    unsigned long long service_sum, latest_unqueued, longest_pair, over_range, longest_prefill, longest_tpot;
};

__global__ __launch_bounds__(kRoofThreads) void k_table_bounds(const uint32_t* __restrict__ tab_prefill,
                                                               const uint32_t* __restrict__ tab_tpot,
                                                               const uint32_t* __restrict__ types, uint32_t n_types,
                                                               const uint32_t* __restrict__ arrival,
                                                               const uint32_t* __restrict__ outlen, uint32_t R,
                                                               TableBounds* __restrict__ out,
                                                               uint32_t* __restrict__ worst_service) {
    unsigned long long sum = 0, latest = 0, pair = 0, over = 0;
    uint32_t top_prefill = 0, top_tpot = 0;
    for (uint32_t r = blockIdx.x * kRoofThreads + threadIdx.x; r < R; r += gridDim.x * kRoofThreads) {
        unsigned long long worst = 0;
        for (uint32_t i = 0; i < n_types; ++i) {
            const size_t at = (size_t)types[i] * R + r;
            const uint32_t prefill = tab_prefill[at], tpot = tab_tpot[at];
            over += (prefill == 0xFFFFFFFFu || tpot == 0xFFFFFFFFu) ? 1ull : 0ull;
            worst = max(worst, (unsigned long long)prefill + (unsigned long long)outlen[r] * tpot);
            top_prefill = max(top_prefill, prefill);
            top_tpot = max(top_tpot, tpot);
        }
        worst_service[r] = (uint32_t)min(worst, 0xFFFFFFFEull);
        sum += min(worst, 1ull << 33);
        latest = max(latest, (unsigned long long)arrival[r] + worst);
        pair = max(pair, (unsigned long long)arrival[r] + worst - arrival[r & ~1u]);
    }
    for (uint32_t dlt = 32u; dlt != 0u; dlt >>= 1) {
        sum += (unsigned long long)__shfl_down((long long)sum, dlt);
        over += (unsigned long long)__shfl_down((long long)over, dlt);
        latest = max(latest, (unsigned long long)__shfl_down((long long)latest, dlt));
        pair = max(pair, (unsigned long long)__shfl_down((long long)pair, dlt));
        top_prefill = max(top_prefill, (uint32_t)__shfl_down((int)top_prefill, dlt));
        top_tpot = max(top_tpot, (uint32_t)__shfl_down((int)top_tpot, dlt));
    }
    if ((threadIdx.x & 63u) == 0u) {
        if (sum) atomicAdd(&out->service_sum, sum);
        if (over) atomicAdd(&out->over_range, over);
        atomicMax(&out->latest_unqueued, latest);
        atomicMax(&out->longest_pair, pair);
        atomicMax(&out->longest_prefill, (unsigned long long)top_prefill);
        atomicMax(&out->longest_tpot, (unsigned long long)top_tpot);
    }
}

// ----------------------------------------------------------------------------------
// reconfiguration cost and end-to-end trace time
// ----------------------------------------------------------------------------------
// Weight transfer time tau(z, g) = W_z / P_g * c_z (Appendix "Serving Simulator", Reconfiguration Cost),
// in whole nanoseconds.  `models` are RoofGroups of which only the model fields are used.
__global__ __launch_bounds__(kRoofThreads) void k_transfer_times(const RoofGroup* __restrict__ models, const double* __restrict__ coef,
                                                                 uint32_t n_models, const double* __restrict__ pcie,
                                                                 uint32_t n_gpus, unsigned long long* __restrict__ tau_ns) {
#pragma clang fp contract(off)
    const uint32_t i = blockIdx.x * kRoofThreads + threadIdx.x;
    if (i >= n_models * n_gpus) return;
    const uint32_t z = i / n_gpus, g = i - z * n_gpus;
    tau_ns[i] = roof_ns((roof_weight_bytes(models[z]) / pcie[g]) * coef[z]);
}

// The same with the descriptions passed in the kernel's arguments (no device copy of them has to exist):
// `a` holds n_models models with their coefficients and the PCIe bandwidth of n_gpus GPU types.
constexpr uint32_t kTransferArgModels = 64, kTransferArgGpus = 16;
struct TransferArgs {
    ap_model model[kTransferArgModels];
    double coef[kTransferArgModels];
    double pcie[kTransferArgGpus];
};
__global__ __launch_bounds__(kRoofThreads) void k_transfer_times_from_args(TransferArgs a, uint32_t n_models, uint32_t n_gpus,
                                                                           unsigned long long* __restrict__ tau_ns) {
#pragma clang fp contract(off)
    const uint32_t i = blockIdx.x * kRoofThreads + threadIdx.x;
    if (i >= n_models * n_gpus) return;
    const uint32_t z = i / n_gpus, g = i - z * n_gpus;
    const ap_model& m = a.model[z];
    RoofGroup o{};
    o.L = m.layers; o.H = m.hidden; o.I = m.intermediate; o.V = m.vocab; o.A = m.heads; o.K = m.kv_heads;
    o.e = (double)m.weight_bits / 8.0;
    tau_ns[i] = roof_ns((roof_weight_bytes(o) / a.pcie[g]) * a.coef[z]);
}

struct TraceTimeParams {
    const unsigned long long* tau_ns;     // [Z][G]
    const ap_placement* plans;            // [C][N_max][Z][G]
    const uint32_t* n_intervals;          // [C]
    const unsigned long long* sched_ns;   // [C]
    const unsigned long long* stale_ns;   // [C][N_max]
    const unsigned long long* serve_ns;   // [C][N_max]
    uint32_t C, N_max, Z, G;
    uint32_t load_changed_only;           // the loading cost over the changed models only (else: every model the new plan deploys)
};

// One thread per candidate: T_total = t_sched(1) + t_serve(1) + sum over i >= 2 of t_stale(i) +
// Reconfig-Cost(sigma_{i-1}, sigma_i) + t_serve(i) (Section 5.1, execution model), where
// Reconfig-Cost = T_term + T_load (Appendix "Serving Simulator", Reconfiguration Cost): T_term is the largest
// transfer time, over the models whose (GPU type, TP, count) tuples changed, on a GPU type the previous plan
// had them on; T_load is the largest transfer time over every model the new plan deploys, on the GPU types it
// deploys them on (the loading-cost equation takes the new plan alone) - or, with load_changed_only, over the
// changed models only; both are zero when no model changed.  Integers throughout.
__global__ __launch_bounds__(kRoofThreads) void k_trace_time(TraceTimeParams p, ap_breakdown* __restrict__ out) {
    const uint32_t c = blockIdx.x * kRoofThreads + threadIdx.x;
    if (c >= p.C) return;
    const uint32_t n = min(max(p.n_intervals[c], 1u), p.N_max);
    const size_t per_plan = (size_t)p.Z * p.G;
    const ap_placement* plans = p.plans + (size_t)c * p.N_max * per_plan;
    unsigned long long stale = 0ull, reconfig = 0ull, serve = p.serve_ns[(size_t)c * p.N_max];
    for (uint32_t i = 1; i < n; ++i) {
        const ap_placement* prev = plans + (size_t)(i - 1u) * per_plan;
        const ap_placement* next = plans + (size_t)i * per_plan;
        unsigned long long term = 0ull, load_changed = 0ull, load_deployed = 0ull;
        bool any_changed = false;
        for (uint32_t z = 0; z < p.Z; ++z) {
            bool changed = false;
            for (uint32_t g = 0; g < p.G; ++g) {
                const ap_placement a = prev[z * p.G + g], b = next[z * p.G + g];
                changed = changed || a.count != b.count || (a.count != 0u && a.tp != b.tp);
            }
            any_changed = any_changed || changed;
            for (uint32_t g = 0; g < p.G; ++g) {
                const unsigned long long tau = p.tau_ns[z * p.G + g];
                if (changed && prev[z * p.G + g].count != 0u) term = max(term, tau);
                if (next[z * p.G + g].count != 0u) {
                    load_deployed = max(load_deployed, tau);
                    if (changed) load_changed = max(load_changed, tau);
                }
            }
        }
        const unsigned long long load = !any_changed ? 0ull : (p.load_changed_only ? load_changed : load_deployed);
        stale += p.stale_ns[(size_t)c * p.N_max + i];
        reconfig += term + load;
        serve += p.serve_ns[(size_t)c * p.N_max + i];
    }
    ap_breakdown r;
    r.sched_ns = p.sched_ns[c];
    r.sum_stale_ns = stale;
    r.sum_reconfig_ns = reconfig;
    r.sum_serve_ns = serve;
    r.total_ns = r.sched_ns + stale + reconfig + serve;
    r.n_intervals = n;
    r.reserved = 0u;
    out[c] = r;
}

}  // namespace

#endif  // AP_ROOFLINE_HPP
