// Candidate-assignment evaluator for MI355X (gfx950): kernels and C ABI.
//
// One workgroup scores one candidate at a time.  The trace is walked in time chunks;
// for every chunk the workgroup
//   (1) counts the chunk's requests per replica        (replica histogram, LDS atomics),
//   (2) turns the counts into offsets                  (wavefront exclusive scans),
//   (3) scatters request indices by replica, stably    (rank inside a wavefront by ballots),
//   (4) replays every replica's queue segment, one wavefront per replica: the B
//       slot-free times live one per lane and persist in LDS between chunks,
//   (5) feeds TTFT / TPOT / E2E of every served request into LDS histograms and
//       per-lane sums.
// After the last chunk the histograms give the p99 values and one 64-byte record is
// written.  Grouping by replica in arrival order is the per-instance queue order of
// Section 8.3 (Setup); the B-slot queue is continuous batching with maximum batch size
// b^max (Section 5.3 "Serving simulator"); the reductions are the per-request
// objectives of Appendix "Discussion and Limitation" (adaptability to diverse serving
// objectives).
//
// Time on the device is 32-bit microseconds relative to the first arrival;
// ap_costmodel_set proves that no finish time can overflow before it enables the path.
//
// This file holds the host side: planning, the workload object and the C ABI.  The kernels are in
// ap_screen.hpp (screening), ap_replay.hpp (fused replay), ap_pipeline.hpp (three-kernel replay) and
// ap_children.hpp (sparse candidates), ap_split.hpp (replicas that differ or come and go: listed and streamed
// part), ap_roofline.hpp (roofline cost tables, trace time) and ap_agentic.hpp (agentic workflows); ap_common.hpp
// has what they share.
#include <mutex>

#include "ap_common.hpp"
#include "ap_screen.hpp"
#include "ap_replay.hpp"
#include "ap_pipeline.hpp"
#include "ap_children.hpp"
#include "ap_split.hpp"
#include "ap_roofline.hpp"
#include "ap_agentic.hpp"

namespace {

// ----------------------------------------------------------------------------------
// host side
// ----------------------------------------------------------------------------------
inline uint32_t align_up(uint32_t v, uint32_t a) { return (v + a - 1u) / a * a; }

// LDS layout for a given chunk size; returns total bytes.
uint32_t plan_lds(EvalParams& p, uint32_t chunk, bool hist16, bool len16) {
    uint32_t off = 3u * kBins * (hist16 ? 2u : 4u);
    p.off_slots = off;  off += align_up(p.M * p.B * 4u, 16u);
    p.off_sorted = off; off += align_up(p.M * 4u, 16u);
    p.off_close = off;  off += align_up((p.M + 1u) * 4u, 16u);
    p.off_cnt = off;    off += align_up(kWaves * (p.M + 1u) * 4u, 16u);
    p.off_qstart = off; off += align_up((p.M + 2u) * 4u, 16u);
    p.off_list = off;   off += align_up(chunk * 2u, 16u);
    p.off_arr = off;    off += chunk * 4u;
    p.off_prompt = off; off += align_up(chunk * (len16 ? 2u : 4u), 16u);
    p.off_out = off;    off += align_up(chunk * (len16 ? 2u : 4u), 16u);
    p.off_misc = off;   off += 64u + 3u * kWaves * 4u;
    p.chunk = chunk;
    return off;
}

using EvalKernel = void (*)(EvalParams, const uint16_t*, ap_metrics*, uint32_t, uint32_t, PendingWord);

EvalKernel eval_kernel(bool hist16, bool len16, bool tabled) {
    static const EvalKernel variants[8] = {
        k_eval_candidates<false, false, false>, k_eval_candidates<true, false, false>,
        k_eval_candidates<false, true, false>,  k_eval_candidates<true, true, false>,
        k_eval_candidates<false, false, true>,  k_eval_candidates<true, false, true>,
        k_eval_candidates<false, true, true>,   k_eval_candidates<true, true, true>};
    return variants[(hist16 ? 1 : 0) + (len16 ? 2 : 0) + (tabled ? 4 : 0)];
}

}  // namespace

constexpr size_t kNominalSumsBytes = 3u * kBins * sizeof(uint32_t) + 3u * sizeof(unsigned long long) + 4u * sizeof(uint32_t);

namespace {
// Every failed device call ends here: HIP keeps the error of a failed call until somebody reads it, and the next,
// unrelated call must not find it.
ap_status device_error() {
    (void)hipGetLastError();
    return AP_ERR_DEVICE;
}

// Device buffers of one roofline computation; freed when the object goes out of scope.
struct RoofBuffers {
    RoofGroup* groups = nullptr;
    unsigned long long* prefill_ns = nullptr;
    unsigned long long* step_ns = nullptr;
    unsigned long long* prefix_ns = nullptr;
    double* weight_bytes = nullptr;
    uint32_t* feasible = nullptr;
    uint32_t* prefill_us = nullptr;
    uint32_t* tpot_us = nullptr;
    uint32_t cap_groups = 0, cap_seq = 0;       // what the table buffers hold; a later computation that fits reuses them
    void release() {
        for (void* q : {(void*)groups, (void*)prefill_ns, (void*)step_ns, (void*)prefix_ns, (void*)weight_bytes,
                        (void*)feasible, (void*)prefill_us, (void*)tpot_us})
            if (q) (void)hipFree(q);
        groups = nullptr; prefill_ns = step_ns = prefix_ns = nullptr; weight_bytes = nullptr; feasible = nullptr;
        prefill_us = tpot_us = nullptr;
        cap_groups = cap_seq = 0;
    }
    ~RoofBuffers() { release(); }
};
}  // namespace

struct ap_workload {
    int device = 0;
    uint32_t R = 0;
    uint64_t base_us = 0;             // first arrival
    uint64_t span_us = 0;             // last arrival - first arrival
    std::vector<int32_t> h_prompt, h_out;
    std::vector<uint32_t> h_arrival;  // relative to base_us (clamped; a span beyond 32 bits is refused anyway)
    uint32_t* d_arrival = nullptr;
    uint32_t* d_prompt = nullptr;
    uint32_t* d_out = nullptr;
    DevReplica* d_rep = nullptr;      // capacity AP_MAX_REPLICAS
    uint32_t* d_tab_prefill = nullptr;  // [T][R] cost tables (ap_costtable_set), kept for the largest T seen
    uint32_t* d_tab_tpot = nullptr;
    size_t tab_entries = 0;
    bool tabled = false;              // the current cost model reads the tables
    RoofBuffers* roof = nullptr;             // device buffers of ap_costtable_set_roofline, kept for the next call
    unsigned char* d_bounds = nullptr;       // TableBounds, then the replica types in use [AP_MAX_REPLICAS]
    uint32_t* d_span = nullptr;       // [R] contention-free service intervals in ticks, valid when screen is set
    uint32_t* d_span_t = nullptr;     // the same, lane-major for the one-wavefront screening kernel
    uint32_t* d_pair = nullptr;       // one word per two requests (eight-wavefront screening kernel, when it fits)
    bool screen_packed = false;       // that kernel reads d_pair instead of d_span
    ap_metrics* d_nominal = nullptr;  // record shared by all contention-free candidates
    unsigned char* d_nominal_sums = nullptr;   // k_nominal_metrics: three histograms of 32-bit counts, then its sums and counters
    uint32_t* d_pending = nullptr;    // [2] "this call has left pending marks", taken in turn by the calls; [2] = candidates replayed
    mutable uint32_t turn = 0;        // which of the two the next call uses
    mutable uint64_t n_scored = 0;    // candidates scored since the cost model was set
    bool has_model = false;
    bool screen = false;              // homogeneous, always-on replicas: screening applies
    bool hist16 = false;              // R < 65536: 16-bit histogram counters
    bool len16 = false;               // every prompt and output length < 65536: 16-bit staging
    EvalParams params{};
    ScreenParams screen_params{};
    uint32_t lds_bytes = 0;
    uint32_t screen_lds_bytes = 0;
    bool screen_wide = false;         // eight wavefronts per candidate (large replica tables)
    uint32_t screen_wide_lds_bytes = 0;
    uint32_t max_grid = 0;
    uint32_t resident_grid = 0;       // workgroups of the replay kernel that fit on the device at once
    uint32_t n_cu = 0;
    // three-kernel replay: request records, scratch for one batch of candidates, launch parameters
    uint4* d_req = nullptr;           // [R] {arrival, prompt_len, out_len, 0}
    unsigned char* d_scratch = nullptr;
    size_t scratch_bytes = 0;
    uint32_t batch = 0;               // candidates per batch
    GroupParams group_params{};
    ReplayParams replay_params{};
    ReduceParams reduce_params{};
    EvalParams reduce_eval{};
    uint32_t group_lds_bytes = 0, replay_lds_bytes = 0, reduce_lds_bytes = 0;
    bool pipeline = false;
    // sparse candidates (ap_parent_set / ap_eval_children)
    uint16_t* d_parent = nullptr;     // [R]
    uint32_t* d_peak = nullptr;       // [AP_MAX_REPLICAS + 1] depth of the parent per replica, then its unknown ids
    uint32_t* d_room = nullptr;       // [AP_MAX_REPLICAS]
    unsigned char* h_stage = nullptr; // pinned: the parent row on its way in, then the depths on their way out
    uint16_t* d_rows = nullptr;       // [max_children][R]
    size_t rows_bytes = 0;
    uint32_t max_children = 0;
    bool has_parent = false;
    ChildParams child_params{};
    // split evaluation (replicas that differ or have windows): listed part replayed, streamed part scored on arrival
    uint2* d_req8 = nullptr;          // [R] {arrival, prompt | out << 16}; only when every length is below 65536
    uint2* d_tab_pair = nullptr;      // [T][R] the cost tables side by side, for the split evaluation of a tabulated model
    size_t tab_pair_entries = 0;
    uint32_t* d_split_tab = nullptr;       // range and kind words [2][AP_MAX_REPLICAS + 1], then the coefficients of every kind
    SplitQueue* d_split_queue = nullptr;   // [AP_MAX_REPLICAS]
    uint32_t* d_split_order = nullptr;     // [AP_MAX_REPLICAS]
    unsigned char* d_split_scratch = nullptr;
    size_t split_scratch_bytes = 0;
    bool split = false;               // the split evaluation runs in front of the general replay
    bool split_expect_lazy = false;   // stream without histograms first
    uint32_t split_batch = 0;         // candidates per batch (what the scratch area holds)
    uint32_t split_lds_bytes = 0, split_lds_bytes_hist = 0;
    uint32_t split_slots = 0;         // B rounded up to 8, 16, 32 or 64
    SplitParams split_params{};
};

typedef void (*split_fn)(SplitParams, const uint16_t*, uint32_t, uint32_t, uint32_t, PendingWord);
static split_fn split_kernel(uint32_t hist_mode, int narrow, bool tabled) {
    static const split_fn variants[12] = {
        k_split_candidates<0u, false, false>, k_split_candidates<1u, false, false>, k_split_candidates<2u, false, false>,
        k_split_candidates<0u, true, false>,  k_split_candidates<1u, true, false>,  k_split_candidates<2u, true, false>,
        k_split_candidates<0u, false, true>,  k_split_candidates<1u, false, true>,  k_split_candidates<2u, false, true>,
        k_split_candidates<0u, true, true>,   k_split_candidates<1u, true, true>,   k_split_candidates<2u, true, true>};
    return variants[hist_mode + (narrow ? 3u : 0u) + (tabled ? 6u : 0u)];
}

typedef void (*replay_lists_fn)(SplitParams, uint32_t, uint32_t);
template <bool kBinsOut, bool kTabled>
static replay_lists_fn replay_lists_kernel_of(uint32_t slots) {
    return slots == 8u ? k_replay_lists<8u, kBinsOut, kTabled> : slots == 16u ? k_replay_lists<16u, kBinsOut, kTabled>
           : slots == 32u ? k_replay_lists<32u, kBinsOut, kTabled> : k_replay_lists<64u, kBinsOut, kTabled>;
}
static replay_lists_fn replay_lists_kernel(uint32_t slots, bool bins_out, bool tabled) {
    if (tabled) return bins_out ? replay_lists_kernel_of<true, true>(slots) : replay_lists_kernel_of<false, true>(slots);
    return bins_out ? replay_lists_kernel_of<true, false>(slots) : replay_lists_kernel_of<false, false>(slots);
}

// The dense path on C rows: screening where it applies, then the exact replay of what is left.
// marked: only rows whose record carries the pending mark are looked at (screening applies).
static PendingWord take_pending_word(const ap_workload* w) {
    const uint32_t t = w->turn;
    w->turn = t ^ 1u;
    return PendingWord{w->d_pending + t, w->d_pending + (t ^ 1u)};
}

static ap_status launch_dense(const ap_workload* w, const uint16_t* d_assign, uint32_t C, ap_metrics* d_out,
                              hipStream_t stream, bool marked, PendingWord flags) {
    if (w->screen) {
        const uint32_t blocks = std::min((C + kScreenWaves - 1u) / kScreenWaves, w->n_cu * 64u);
        // rows start on 4-byte boundaries when R is even and the batch itself does
        const bool aligned = (w->R % 2u == 0u) && (reinterpret_cast<uintptr_t>(d_assign) % 4u == 0u);
        typedef void (*screen_fn)(ScreenParams, const uint16_t*, ap_metrics*, uint32_t, PendingWord);
        if (w->screen_wide) {
            static const screen_fn wide[8] = {
                k_screen_candidates_wide<false, false, false>, k_screen_candidates_wide<true, false, false>,
                k_screen_candidates_wide<false, true, false>,  k_screen_candidates_wide<true, true, false>,
                k_screen_candidates_wide<false, false, true>,  k_screen_candidates_wide<true, false, true>,
                k_screen_candidates_wide<false, true, true>,   k_screen_candidates_wide<true, true, true>};
            // one candidate per workgroup while the grid stays moderate: workgroups finish at different
            // times, and the hardware's queue of waiting workgroups balances that better than fixed shares
            // marked: runs of candidates per workgroup (at most one per thread), few workgroups
            const uint32_t grid = marked ? std::max((C + kWideThreads - 1u) / kWideThreads, std::min(C, w->n_cu * 4u))
                                         : std::min(C, w->n_cu * 64u);
            hipLaunchKernelGGL(wide[(aligned ? 1 : 0) + (w->screen_packed ? 2 : 0) + (marked ? 4 : 0)], dim3(grid),
                               dim3(kWideThreads), w->screen_wide_lds_bytes, stream, w->screen_params, d_assign, d_out, C, flags);
        } else {
            static const screen_fn narrow[4] = {k_screen_candidates<false, false>, k_screen_candidates<true, false>,
                                                k_screen_candidates<false, true>, k_screen_candidates<true, true>};
            const uint32_t grid = marked ? std::max((C + kScreenThreads - 1u) / kScreenThreads, std::min(blocks, w->n_cu * 8u))
                                         : blocks;
            hipLaunchKernelGGL(narrow[(aligned ? 1 : 0) + (marked ? 2 : 0)], dim3(grid), dim3(kScreenThreads),
                               w->screen_lds_bytes, stream, w->screen_params, d_assign, d_out, C, flags);
        }
        if (hipGetLastError() != hipSuccess) return device_error();
    }
    if (w->split && !marked) {
        // the listed / streamed evaluation, a batch of candidates at a time; what it hands back carries the pending mark
        const SplitParams& sp = w->split_params;
        const replay_lists_fn replay_lean = replay_lists_kernel(w->split_slots, false, w->tabled);
        const replay_lists_fn replay_bins = replay_lists_kernel(w->split_slots, true, w->tabled);
        // batches of equal size (whole wavefronts of the list replay), none above what the scratch area holds
        const uint32_t n_batches = (C + w->split_batch - 1u) / w->split_batch;
        const uint32_t per_batch = std::min(w->split_batch, ((C + n_batches - 1u) / n_batches + 63u) / 64u * 64u);
        for (uint32_t c0 = 0; c0 < C; c0 += per_batch) {
            const uint32_t n = std::min(per_batch, C - c0);
            const uint32_t grid = std::min(n, w->n_cu * 16u);
            // First without histograms where the candidates are expected to be settled by penalty, or where nothing is
            // streamed at all; then with histograms, for every candidate or for those the first pass marked.
            const int narrow = sp.M <= 64u ? 1 : 0;
            const bool plain_first = w->split_expect_lazy || sp.any_streamed == 0u;
            if (plain_first)
                hipLaunchKernelGGL(split_kernel(0u, narrow, w->tabled), dim3(grid), dim3(kSplitThreads), w->split_lds_bytes, stream, sp,
                                   d_assign, c0, n, 0u, flags);
            if (sp.any_streamed != 0u)
                hipLaunchKernelGGL(split_kernel(sp.wide ? 2u : 1u, narrow, w->tabled), dim3(grid), dim3(kSplitThreads),
                                   w->split_lds_bytes_hist, stream, sp, d_assign, c0, n, plain_first ? 1u : 0u, flags);
            // the list replay: where most candidates are settled by penalty, those go through the variant that
            // leaves no bins, and the wavefronts of the other variant find the few that remain
            if (sp.n_queues != 0u) {
                const dim3 groups(sp.n_queues * ((n + kReplayListThreads - 1u) / kReplayListThreads));
                if (w->split_expect_lazy)
                    hipLaunchKernelGGL(replay_lean, groups, dim3(kReplayListThreads), 0, stream, sp, n, 1u);
                hipLaunchKernelGGL(replay_bins, groups, dim3(kReplayListThreads), 0, stream, sp, n,
                                   w->split_expect_lazy ? 2u : 0u);
            }
            hipLaunchKernelGGL(sp.wide ? k_merge_candidates<false> : k_merge_candidates<true>,
                               dim3(std::min(n, w->n_cu * 8u)), dim3(kThreads), w->reduce_lds_bytes,
                               stream, w->reduce_eval, sp, d_out, c0, n, flags);
        }
        if (hipGetLastError() != hipSuccess) return device_error();
    }
    const uint32_t pending_only = (w->screen || (w->split && !marked)) ? 1u : 0u;
    if (w->pipeline) {
        for (uint32_t c0 = 0; c0 < C; c0 += w->batch) {
            const uint32_t n = std::min(w->batch, C - c0);
            hipLaunchKernelGGL(k_group_requests, dim3(n), dim3(kGroupThreads), w->group_lds_bytes, stream, w->group_params,
                               d_assign, d_out, c0, n, pending_only);
            const uint32_t n_wg = (n * w->params.M + kReplayThreads - 1u) / kReplayThreads;
            hipLaunchKernelGGL(k_replay_queues, dim3(n_wg), dim3(kReplayThreads), w->replay_lds_bytes, stream,
                               w->replay_params, d_out, c0, n, pending_only);
            hipLaunchKernelGGL(w->hist16 ? k_reduce_candidates<true> : k_reduce_candidates<false>, dim3(n), dim3(kThreads),
                               w->reduce_lds_bytes, stream, w->reduce_eval, w->reduce_params, d_out, c0, n, pending_only);
        }
        if (hipGetLastError() != hipSuccess) return device_error();
        return AP_OK;
    }
    // After screening, most workgroups only find out that nothing is left for them: as many as can be
    // resident at once look at all the records together.
    const uint32_t grid = std::min(C, pending_only ? w->resident_grid : w->max_grid);
    hipLaunchKernelGGL(eval_kernel(w->hist16, w->len16, w->tabled), dim3(grid), dim3(kThreads), w->lds_bytes, stream, w->params,
                       d_assign, d_out, C, pending_only, flags);
    if (hipGetLastError() != hipSuccess) return device_error();
    return AP_OK;
}

extern "C" {

const char* ap_status_str(ap_status s) {
    switch (s) {
        case AP_OK: return "ok";
        case AP_ERR_INVALID: return "invalid argument";
        case AP_ERR_RANGE: return "capacity of the device path exceeded";
        case AP_ERR_ALLOC: return "allocation failed";
        case AP_ERR_DEVICE: return "HIP call failed";
        case AP_ERR_STATE: return "no cost model (or, for children, no parent) set";
    }
    return "unknown status";
}

uint32_t ap_hist_bin(uint64_t v) {
    if (v < 128u) return (uint32_t)v;
    uint32_t e = 0;
    for (uint64_t t = v; t > 1u; t >>= 1) ++e;         // floor(log2 v)
    if (e > 37u) return kBins - 1u;
    return ((e - 6u) << 7) | (uint32_t)((v >> (e - 7u)) & 127u);
}

uint64_t ap_hist_lower(uint32_t bin) {
    if (bin < 128u) return bin;
    return (uint64_t)(128u | (bin & 127u)) << ((bin >> 7) - 1u);
}

ap_status ap_workload_create(const uint64_t* arrival_us, const int32_t* prompt_len, const int32_t* out_len,
                             uint32_t R, ap_workload** out) {
    if (!arrival_us || !prompt_len || !out_len || !out || R == 0) return AP_ERR_INVALID;
    for (uint32_t r = 0; r < R; ++r) {
        if (prompt_len[r] < 1 || out_len[r] < 1) return AP_ERR_INVALID;
        if (r && arrival_us[r] < arrival_us[r - 1]) return AP_ERR_INVALID;
    }
    ap_workload* w = new (std::nothrow) ap_workload;
    if (!w) return AP_ERR_ALLOC;
    std::vector<uint32_t> rel;
    try {
        w->h_prompt.assign(prompt_len, prompt_len + R);
        w->h_out.assign(out_len, out_len + R);
        rel.resize(R);
    } catch (const std::bad_alloc&) {
        delete w;
        return AP_ERR_ALLOC;
    }
    w->R = R;
    w->len16 = true;
    for (uint32_t r = 0; r < R; ++r) w->len16 = w->len16 && prompt_len[r] < 65536 && out_len[r] < 65536;
    w->base_us = arrival_us[0];
    w->span_us = arrival_us[R - 1] - arrival_us[0];
    // relative 32-bit arrivals; a span that does not fit is refused later by ap_costmodel_set
    for (uint32_t r = 0; r < R; ++r) rel[r] = (uint32_t)std::min<uint64_t>(arrival_us[r] - w->base_us, kNever);
    w->h_arrival = rel;

    ap_status st = AP_OK;
    if (hipGetDevice(&w->device) != hipSuccess) st = AP_ERR_DEVICE;
    const size_t bytes = (size_t)R * 4u;
    const size_t padded = ((size_t)R + kScreenBlock - 1u) / kScreenBlock * kScreenBlock * 4u;
    if (st == AP_OK && (hipMalloc(&w->d_arrival, bytes) != hipSuccess || hipMalloc(&w->d_prompt, bytes) != hipSuccess ||
                        hipMalloc(&w->d_out, bytes) != hipSuccess ||
                        hipMalloc(&w->d_rep, sizeof(DevReplica) * AP_MAX_REPLICAS) != hipSuccess ||
                        hipMalloc(&w->d_span, bytes) != hipSuccess ||
                        hipMalloc(&w->d_span_t, padded) != hipSuccess ||
                        hipMalloc(&w->d_pair, ((size_t)R + 1u) / 2u * 4u) != hipSuccess ||
                        hipMalloc(&w->d_nominal, sizeof(ap_metrics)) != hipSuccess ||
                        hipMalloc(&w->d_nominal_sums, kNominalSumsBytes) != hipSuccess ||
                        hipMalloc(&w->d_pending, 4u * sizeof(uint32_t)) != hipSuccess))
        st = AP_ERR_ALLOC;
    if (st == AP_OK && hipMemset(w->d_pending, 0, 4u * sizeof(uint32_t)) != hipSuccess) st = AP_ERR_DEVICE;
    std::vector<uint4> recs;
    if (st == AP_OK) {
        try {
            recs.resize(R);
        } catch (const std::bad_alloc&) {
            st = AP_ERR_ALLOC;
        }
    }
    if (st == AP_OK) {
        for (uint32_t r = 0; r < R; ++r) recs[r] = make_uint4(rel[r], (uint32_t)prompt_len[r], (uint32_t)out_len[r], 0u);
        if (hipMalloc(&w->d_req, sizeof(uint4) * (size_t)R) != hipSuccess) st = AP_ERR_ALLOC;
        else if (hipMemcpy(w->d_req, recs.data(), sizeof(uint4) * (size_t)R, hipMemcpyHostToDevice) != hipSuccess)
            st = AP_ERR_DEVICE;
    }
    if (st == AP_OK && w->len16) {
        // arrival and both lengths of a request in 8 bytes, for the kernels that read whole records
        std::vector<uint2> packed;
        try {
            packed.assign((size_t)R + 1u, make_uint2(0u, 0u));       // one spare record: pairs of records are read at once
        } catch (const std::bad_alloc&) {
            st = AP_ERR_ALLOC;
        }
        if (st == AP_OK) {
            for (uint32_t r = 0; r < R; ++r) packed[r] = make_uint2(rel[r], (uint32_t)prompt_len[r] | ((uint32_t)out_len[r] << 16));
            if (hipMalloc(&w->d_req8, sizeof(uint2) * ((size_t)R + 1u)) != hipSuccess) st = AP_ERR_ALLOC;
            else if (hipMemcpy(w->d_req8, packed.data(), sizeof(uint2) * ((size_t)R + 1u), hipMemcpyHostToDevice) != hipSuccess)
                st = AP_ERR_DEVICE;
        }
    }
    if (st == AP_OK && (hipMemcpy(w->d_arrival, rel.data(), bytes, hipMemcpyHostToDevice) != hipSuccess ||
                        hipMemcpy(w->d_prompt, prompt_len, bytes, hipMemcpyHostToDevice) != hipSuccess ||
                        hipMemcpy(w->d_out, out_len, bytes, hipMemcpyHostToDevice) != hipSuccess))
        st = AP_ERR_DEVICE;
    if (st != AP_OK) {
        (void)hipGetLastError();
        ap_workload_destroy(w);
        return st;
    }
    *out = w;
    return AP_OK;
}

// Plan of the split evaluation (ap_split.hpp) - replicas that differ or have windows, crowded traces, tables too
// small for the one-wavefront screen; linear cost models (rep_type == nullptr) and tabulated ones:
// the index ranges of every replica, the bound D on requests in service that started on arrival, the
// scratch area for one batch of candidates.  Leaves w->split false where the path does not apply.
// rep_type: the tabulated cost model (replica m reads row rep_type[m] of the tables, which are on the device by
// now); table_longest_prefill / table_longest_tpot are then the largest entries of the rows in use.
static ap_status plan_split(ap_workload* w, const std::vector<DevReplica>& dev, const ap_replica* replicas,
                            const std::vector<uint32_t>& kinds, const std::vector<uint32_t>& worst_service,
                            const std::vector<uint64_t>& kind_sum, const std::vector<uint64_t>& kind_longest,
                            uint64_t latest_finish_bound, const uint32_t* rep_type, uint64_t table_longest_prefill,
                            uint64_t table_longest_tpot) {
    const uint32_t R = w->R, M = w->params.M, B = w->params.B;
    if (!w->d_req8) return AP_OK;                            // request records with 16-bit lengths only
    const bool tabled = rep_type != nullptr;
    const bool wide = R >= 65536u;                           // two range words per replica, 32-bit histogram counts
    // The kernels multiply with 24-bit factors and add up a tile's sixteen latencies per lane in 32 bits.
    uint64_t longest_tpot = table_longest_tpot, longest_prefill = table_longest_prefill;
    for (uint32_t m = 0; m < M && !tabled; ++m) {
        if (replicas[m].prefill_per_tok_us >= (1u << 24) || replicas[m].decode_per_kctx_us >= (1u << 24)) return AP_OK;
        longest_tpot = std::max<uint64_t>(longest_tpot, (uint64_t)replicas[m].decode_base_us + 64ull * replicas[m].decode_per_kctx_us);
        longest_prefill = std::max<uint64_t>(longest_prefill, (uint64_t)replicas[m].prefill_base_us + 65535ull * replicas[m].prefill_per_tok_us);
    }
    if (longest_tpot >= (1u << 24)) return AP_OK;
    for (uint32_t m = 0; m < M && tabled; ++m)
        if (rep_type[m] >= 1024u) return AP_OK;              // the type rides in ten bits of a tile word
    for (uint32_t r = 0; r < R; ++r)
        if (worst_service[r] >= (1u << 28)) return AP_OK;
    std::vector<uint32_t> depth_from;                        // depth_from[i] = max over r >= i of D(r); [R] = 0
    std::vector<uint32_t> tab;                               // range words, kind words, coefficients
    std::vector<SplitQueue> queue;
    std::vector<uint32_t> order;
    try {
        depth_from.assign((size_t)R + 1u, 0u);
        tab.assign(3u * (AP_MAX_REPLICAS + 1u) + 4u * kinds.size(), 0u);
        queue.resize(M);
        // D(r): sweep in arrival order over a min-heap of the finish times of requests that start on arrival
        std::vector<uint64_t> heap;
        heap.reserve(1024);
        for (uint32_t r = 0; r < R; ++r) {
            const uint64_t a = w->h_arrival[r];
            while (!heap.empty() && heap.front() <= a) {
                std::pop_heap(heap.begin(), heap.end(), std::greater<uint64_t>());
                heap.pop_back();
            }
            heap.push_back(a + worst_service[r]);
            std::push_heap(heap.begin(), heap.end(), std::greater<uint64_t>());
            depth_from[r] = (uint32_t)std::min<size_t>(heap.size(), kNever);
        }
    } catch (const std::bad_alloc&) {
        return AP_ERR_ALLOC;
    }
    for (uint32_t r = R; r-- > 0u;) depth_from[r] = std::max(depth_from[r], depth_from[r + 1u]);

    // The streamed part of a replica may begin where the bound leaves an eighth of the slots to the listed part.
    const uint32_t reserve = B / 8u;
    const uint32_t i_calm = (uint32_t)(std::partition_point(depth_from.begin(), depth_from.end(),
                                                            [&](uint32_t d) { return d + reserve > B; }) - depth_from.begin());
    const uint32_t* arr = w->h_arrival.data();
    uint32_t longest_list = 0;
    uint64_t expect_rejected = 0;
    bool any_streamed = false;
    for (uint32_t m = 0; m < M; ++m) {
        const DevReplica& d = dev[m];
        const uint32_t i_on = (uint32_t)(std::lower_bound(arr, arr + R, d.t_on) - arr);
        const uint32_t i_off = (uint32_t)(std::lower_bound(arr, arr + R, d.t_off) - arr);
        // which kind of replica this is (its service times: mean and longest)
        size_t ki = 0;
        for (size_t k = 0; k < kinds.size(); ++k)
            if (tabled ? rep_type[kinds[k]] == rep_type[m]
                       : (replicas[kinds[k]].prefill_base_us == replicas[m].prefill_base_us &&
                          replicas[kinds[k]].prefill_per_tok_us == replicas[m].prefill_per_tok_us &&
                          replicas[kinds[k]].decode_base_us == replicas[m].decode_base_us &&
                          replicas[kinds[k]].decode_per_kctx_us == replicas[m].decode_per_kctx_us))
                ki = k;
        // The backlog a replica finds when it comes up is about its share of the requests so far; served B at a
        // time it is gone after so many mean service times, and the last of it after one longest service more.
        // Twice that is where the streamed part begins - a guess that only decides how often the list replay has
        // to hand a candidate back, never a result.
        uint32_t i_list = 0;
        if (i_on > 0u) {
            const double mean_service = (double)kind_sum[ki] / R;
            const double drain = 2.0 * (((double)i_on / M) / B + 1.0) * mean_service + (double)kind_longest[ki];
            const uint64_t t_target = (uint64_t)d.t_on + (uint64_t)std::min(drain, 4.0e9);
            i_list = (uint32_t)(std::lower_bound(arr, arr + R, (uint32_t)std::min<uint64_t>(t_target, kNever)) - arr);
        }
        i_list = std::min(std::max(i_list, i_calm), i_off);
        tab[m] = wide ? i_list : (i_list | (i_off << 16));
        tab[AP_MAX_REPLICAS + 1u + m] = i_off;
        tab[2u * (AP_MAX_REPLICAS + 1u) + m] = tabled ? rep_type[m] : (uint32_t)ki;
        any_streamed = any_streamed || i_list < i_off;
        SplitQueue q{};
        q.a = d.a; q.b = d.b; q.c = d.c; q.d = d.d; q.t_on = d.t_on; q.t_off = d.t_off;
        q.i_list = i_list;
        q.t_split = i_list < i_off ? arr[i_list] : kNever;
        q.allow_busy = i_list < i_off ? B - std::min(B, depth_from[i_list]) : 0u;
        queue[m] = q;
        longest_list = std::max(longest_list, i_list);
        expect_rejected += R - i_off;
    }
    tab[M] = 0u;                                             // unknown replica ids: rejected on arrival
    tab[AP_MAX_REPLICAS + 1u + M] = 0u;
    tab[2u * (AP_MAX_REPLICAS + 1u) + M] = 0u;
    for (size_t k = 0; k < kinds.size() && !tabled; ++k) {
        uint32_t* co = &tab[3u * (AP_MAX_REPLICAS + 1u) + 4u * k];
        co[0] = replicas[kinds[k]].prefill_base_us; co[1] = replicas[kinds[k]].prefill_per_tok_us;
        co[2] = replicas[kinds[k]].decode_base_us;  co[3] = replicas[kinds[k]].decode_per_kctx_us;
    }
    for (uint32_t m = 0; m < M; ++m)
        if (queue[m].i_list > 0u) order.push_back(m);
    std::stable_sort(order.begin(), order.end(), [&](uint32_t x, uint32_t y) { return queue[x].i_list > queue[y].i_list; });

    SplitParams sp{};
    sp.R = R; sp.M = M; sp.B = B; sp.key_bits = w->params.key_bits;
    sp.n_tiles = (R + kTile - 1u) / kTile;
    sp.n_list_tiles = (longest_list + kTile - 1u) / kTile;
    sp.tile_cap = align_up(std::min(kTile, R) + 7u * std::min(M, std::min(kTile, R)), 8u);
    sp.n_queues = (uint32_t)order.size();
    sp.slo_ttft = w->params.slo_ttft;
    sp.slo_tpot = w->params.slo_tpot;
    // The p99 values are the penalty latency once R - k99 + 1 requests are rejected, if no served latency can
    // reach the penalty's bin: all of them lie below the bound on finish times of the range proof.
    const bool penalty_on_top = w->params.penalty_bin > ap_hist_bin(latest_finish_bound);
    sp.lazy_from = penalty_on_top ? R - w->params.k99 + 1u : kNever;
    sp.all_within = (longest_prefill <= w->params.slo_ttft && longest_tpot <= w->params.slo_tpot) ? 1u : 0u;
    sp.wide = wide ? 1u : 0u;
    sp.any_streamed = any_streamed ? 1u : 0u;
    sp.hist_words = wide ? 3u * kBins : 3u * kBins / 2u;
    // LDS of the streaming kernel
    uint32_t off = 0;
    const uint32_t hist_bytes = sp.hist_words * 4u;
    sp.off_range = off; off += align_up((M + 1u) * 4u, 16u);
    sp.off_range_off = off; off += wide ? align_up((M + 1u) * 4u, 16u) : 0u;
    sp.off_kind = off;  off += align_up((M + 1u) * 4u, 16u);
    sp.off_coef = off;  off += (uint32_t)kinds.size() * 16u;
    sp.off_acc = off;   off += 64u;
    sp.off_wave = off;
    uint32_t wb = 0;
    wb += align_up(M * 4u, 16u);            sp.w_pos = wb;
    wb += align_up(M * 4u, 16u);            sp.w_queue = wb;
    wb += kTile * (M <= 64u ? 2u : 4u);     sp.w_list = wb;
    wb += align_up(sp.tile_cap * 2u, 16u);  sp.w_same = wb;
    wb += align_up(M * 8u, 16u);            sp.w_tile = wb;
    wb += align_up((M + 1u) * 4u, 16u);
    sp.wave_bytes = wb;
    off += kSplitWaves * wb;
    sp.off_hist = off;
    int lds_cap = 0;
    if (hipDeviceGetAttribute(&lds_cap, hipDeviceAttributeMaxSharedMemoryPerBlock, w->device) != hipSuccess) return device_error();
    if (off + hist_bytes > (uint32_t)lds_cap) return AP_OK;  // a replica table that large stays with the general replay
    w->split_lds_bytes = off;
    w->split_lds_bytes_hist = off + hist_bytes;
    const int narrow = M <= 64u ? 1 : 0;
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(split_kernel(0u, narrow, tabled)),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)off) != hipSuccess ||
        hipFuncSetAttribute(reinterpret_cast<const void*>(split_kernel(wide ? 2u : 1u, narrow, tabled)),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)(off + hist_bytes)) != hipSuccess) {
        (void)hipGetLastError();
        return device_error();
    }
    w->split_slots = B <= 8u ? 8u : B <= 16u ? 16u : B <= 32u ? 32u : 64u;

    // scratch for one batch of candidates: lists, run descriptors, partial records, histograms
    const size_t per_cand = (size_t)sp.n_list_tiles * sp.tile_cap * (2u + 8u) + (size_t)sp.n_list_tiles * (M + 1u) * 4u +
                            sizeof(SplitPartial) + hist_bytes;
    if (per_cand > ((size_t)8 << 30) / 64u) return AP_OK;       // a trace so long that 64 candidates' lists take over 8 GiB
    uint32_t batch = (uint32_t)std::min<size_t>(16384u, std::max<size_t>(64u, ((size_t)4 << 30) / per_cand));
    batch = batch / 64u * 64u;
    auto carve = [](size_t& at, size_t bytes) { const size_t here = at; at = (at + bytes + 255u) / 256u * 256u; return here; };
    size_t total = 0, o_lists = 0, o_bins = 0, o_desc = 0, o_part = 0, o_hist = 0;
    for (;; batch = std::max(64u, batch / 2u / 64u * 64u)) {        // a device short of memory gets smaller batches
        total = 0;
        o_lists = carve(total, (size_t)batch * sp.n_list_tiles * sp.tile_cap * 2u);
        o_bins = carve(total, (size_t)batch * sp.n_list_tiles * sp.tile_cap * 8u);
        o_desc = carve(total, (size_t)batch * sp.n_list_tiles * (M + 1u) * 4u);
        o_part = carve(total, (size_t)batch * sizeof(SplitPartial));
        o_hist = carve(total, (size_t)batch * hist_bytes);
        if (total <= w->split_scratch_bytes) break;
        if (w->d_split_scratch && hipFree(w->d_split_scratch) != hipSuccess) return device_error();
        w->d_split_scratch = nullptr;
        w->split_scratch_bytes = 0;
        if (hipMalloc(&w->d_split_scratch, total) == hipSuccess) {
            w->split_scratch_bytes = total;
            break;
        }
        (void)hipGetLastError();
        w->d_split_scratch = nullptr;
        if (batch == 64u) return AP_OK;                         // no room for the lists: the general replay scores the calls
    }
    const size_t tab_bytes = 4u * (3u * (AP_MAX_REPLICAS + 1u) + 4u * (size_t)AP_MAX_REPLICAS + 4u);
    if ((!w->d_split_tab && hipMalloc(&w->d_split_tab, tab_bytes) != hipSuccess) ||
        (!w->d_split_queue && hipMalloc(&w->d_split_queue, sizeof(SplitQueue) * AP_MAX_REPLICAS) != hipSuccess) ||
        (!w->d_split_order && hipMalloc(&w->d_split_order, sizeof(uint32_t) * AP_MAX_REPLICAS) != hipSuccess)) {
        (void)hipGetLastError();
        return AP_ERR_ALLOC;
    }
    if (hipMemcpy(w->d_split_tab, tab.data(), 4u * tab.size(), hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(w->d_split_queue, queue.data(), sizeof(SplitQueue) * M, hipMemcpyHostToDevice) != hipSuccess ||
        (!order.empty() &&
         hipMemcpy(w->d_split_order, order.data(), sizeof(uint32_t) * order.size(), hipMemcpyHostToDevice) != hipSuccess) ||
        hipFuncSetAttribute(wide ? reinterpret_cast<const void*>(&k_merge_candidates<false>)
                                 : reinterpret_cast<const void*>(&k_merge_candidates<true>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)w->reduce_lds_bytes) != hipSuccess) {
        (void)hipGetLastError();
        return device_error();
    }
    sp.req8 = w->d_req8;
    sp.tab.range = w->d_split_tab;
    sp.tab.range_off = w->d_split_tab + (AP_MAX_REPLICAS + 1u);
    sp.tab.kind = w->d_split_tab + 2u * (AP_MAX_REPLICAS + 1u);
    sp.tab.coef = reinterpret_cast<const uint4*>(w->d_split_tab + 3u * (AP_MAX_REPLICAS + 1u));
    sp.tab.n_kinds = tabled ? 0u : (uint32_t)kinds.size();
    sp.tab_pair = nullptr;
    if (tabled) {
        size_t entries = 0;                                  // rows up to the highest type in use
        for (uint32_t m = 0; m < M; ++m) entries = std::max(entries, ((size_t)rep_type[m] + 1u) * R);
        if (entries > w->tab_pair_entries) {
            if (w->d_tab_pair && hipFree(w->d_tab_pair) != hipSuccess) return device_error();
            w->d_tab_pair = nullptr;
            w->tab_pair_entries = 0;
            if (hipMalloc(&w->d_tab_pair, entries * sizeof(uint2)) != hipSuccess) {
                (void)hipGetLastError();
                return AP_OK;                                // no room: the general replay scores the calls
            }
            w->tab_pair_entries = entries;
        }
        hipLaunchKernelGGL(k_pair_tables, dim3((uint32_t)std::min<size_t>(4096u, (entries + kThreads - 1u) / kThreads)),
                           dim3(kThreads), 0, nullptr, w->d_tab_prefill, w->d_tab_tpot, w->d_tab_pair, entries);
        if (hipGetLastError() != hipSuccess || hipDeviceSynchronize() != hipSuccess) return device_error();
        sp.tab_pair = w->d_tab_pair;
    }
    sp.queue = w->d_split_queue;
    sp.order = w->d_split_order;
    sp.lists = reinterpret_cast<uint16_t*>(w->d_split_scratch + o_lists);
    sp.bins = reinterpret_cast<uint2*>(w->d_split_scratch + o_bins);
    sp.desc = reinterpret_cast<uint32_t*>(w->d_split_scratch + o_desc);
    sp.part = reinterpret_cast<SplitPartial*>(w->d_split_scratch + o_part);
    sp.hist = reinterpret_cast<uint32_t*>(w->d_split_scratch + o_hist);
    w->split_params = sp;
    w->split_batch = batch;
    // stream without histograms first when an even spread of the requests over the replicas would reject enough
    w->split_expect_lazy = penalty_on_top && expect_rejected / M >= sp.lazy_from;
    w->split = true;
    return AP_OK;
}

// Shared by ap_costmodel_set (rep_type == nullptr: the coefficients of `replicas` apply) and
// ap_costtable_set (replica m is of type rep_type[m] < T and the HOST tables [T][R] apply; the
// coefficients are ignored).
// tab_prefill == nullptr with rep_type set: the tables are in the workload's device buffers already
// (ap_costtable_set_roofline) and the bounds come from a reduction over them.
static ap_status set_cost_model_checked(ap_workload* w, const ap_replica* replicas, uint32_t M, uint32_t B, const ap_slo* slo,
                                        const uint32_t* rep_type, const uint32_t* tab_prefill, const uint32_t* tab_tpot,
                                        uint32_t T);

static ap_status set_cost_model(ap_workload* w, const ap_replica* replicas, uint32_t M, uint32_t B, const ap_slo* slo,
                                const uint32_t* rep_type, const uint32_t* tab_prefill, const uint32_t* tab_tpot, uint32_t T) {
    try {                                                   // host containers allocate: nothing may leave through the C ABI
        return set_cost_model_checked(w, replicas, M, B, slo, rep_type, tab_prefill, tab_tpot, T);
    } catch (const std::bad_alloc&) {
        if (w) w->has_model = false;
        return AP_ERR_ALLOC;
    }
}

static ap_status set_cost_model_checked(ap_workload* w, const ap_replica* replicas, uint32_t M, uint32_t B, const ap_slo* slo,
                                        const uint32_t* rep_type, const uint32_t* tab_prefill, const uint32_t* tab_tpot,
                                        uint32_t T) {
    if (!w || !replicas || !slo || M == 0 || B == 0) return AP_ERR_INVALID;
    const bool tabled = rep_type != nullptr;
    const bool on_device = tabled && tab_prefill == nullptr;
    for (uint32_t m = 0; m < M; ++m)
        if (replicas[m].t_on_us > replicas[m].t_off_us) return AP_ERR_INVALID;
    if (M > AP_MAX_REPLICAS || B > AP_MAX_SLOTS) return AP_ERR_RANGE;

    // ---- range proof for 32-bit relative time ------------------------------------------
    // Every start is at most max(latest arrival, latest t_on of a replica that can serve)
    // plus the total of all earlier service on that replica; bound the latter by the sum
    // over requests of their largest service time on any replica.
    const uint64_t limit = (uint64_t)kNever - 1u;
    uint64_t latest = w->span_us;
    for (uint32_t m = 0; m < M; ++m) {
        const ap_replica& rp = replicas[m];
        if (rp.t_on_us >= rp.t_off_us || rp.t_on_us <= w->base_us) continue;   // never serves / already on
        latest = std::max(latest, rp.t_on_us - w->base_us);
    }
    if (latest > limit) return AP_ERR_RANGE;
    // distinct kinds of replica (coefficient sets, or types with tables), each by its first replica
    std::vector<uint32_t> kinds;
    for (uint32_t m = 0; m < M; ++m) {
        bool seen = false;
        for (uint32_t k : kinds)
            seen = seen || (tabled ? rep_type[k] == rep_type[m]
                                   : (replicas[k].prefill_base_us == replicas[m].prefill_base_us &&
                                      replicas[k].prefill_per_tok_us == replicas[m].prefill_per_tok_us &&
                                      replicas[k].decode_base_us == replicas[m].decode_base_us &&
                                      replicas[k].decode_per_kctx_us == replicas[m].decode_per_kctx_us));
        if (!seen) kinds.push_back(m);
    }
    // prefill time and time per token of request r on the kind whose first replica is k
    auto host_cost = [&](uint32_t k, uint32_t r, uint64_t& prefill, uint64_t& tpot) {
        if (tabled) {
            prefill = tab_prefill[(size_t)rep_type[k] * w->R + r];
            tpot = tab_tpot[(size_t)rep_type[k] * w->R + r];
        } else {
            // each term stays far below 2^64: coefficients < 2^32, lengths < 2^31
            const uint64_t prompt = (uint64_t)w->h_prompt[r];
            prefill = (uint64_t)replicas[k].prefill_base_us + (uint64_t)replicas[k].prefill_per_tok_us * prompt;
            tpot = (uint64_t)replicas[k].decode_base_us + (uint64_t)replicas[k].decode_per_kctx_us * ((prompt + 1023u) >> 10);
        }
    };
    uint64_t total = latest;
    uint64_t table_longest_prefill = 0, table_longest_tpot = 0;   // tabulated: the largest entries of the rows in use
    uint64_t latest_unqueued = 0;      // latest finish if nobody ever waited (arrival + service)
    uint64_t longest_pair = 0;         // longest time from the arrival of request 2q to the unqueued finish of 2q or 2q+1
    uint64_t service_sum = 0;
    std::vector<uint32_t> worst_service;            // per request: its longest service time over the kinds of replica
    std::vector<uint64_t> kind_sum, kind_longest;   // per kind: all service times added up, and the longest
    try {
        worst_service.resize(w->R);
        kind_sum.assign(kinds.size(), 0u);
        kind_longest.assign(kinds.size(), 0u);
    } catch (const std::bad_alloc&) {
        return AP_ERR_ALLOC;
    }
    if (on_device) {
        if (hipSetDevice(w->device) != hipSuccess) return device_error();
        std::vector<uint32_t> in_use;
        try {
            for (uint32_t k : kinds) in_use.push_back(rep_type[k]);
        } catch (const std::bad_alloc&) {
            return AP_ERR_ALLOC;
        }
        TableBounds bounds{};
        TableBounds* d_bounds = reinterpret_cast<TableBounds*>(w->d_bounds);
        uint32_t* d_in_use = reinterpret_cast<uint32_t*>(w->d_bounds + sizeof(TableBounds));
        if (hipMemcpy(d_bounds, &bounds, sizeof(bounds), hipMemcpyHostToDevice) != hipSuccess ||
            hipMemcpy(d_in_use, in_use.data(), 4u * in_use.size(), hipMemcpyHostToDevice) != hipSuccess) {
            (void)hipGetLastError();
            return device_error();
        }
        const uint32_t blocks = std::max(1u, std::min(1024u, (w->R + kRoofThreads - 1u) / kRoofThreads));
        hipLaunchKernelGGL(k_table_bounds, dim3(blocks), dim3(kRoofThreads), 0, nullptr, w->d_tab_prefill, w->d_tab_tpot, d_in_use,
                           (uint32_t)in_use.size(), w->d_arrival, w->d_out, w->R, d_bounds, w->d_span);
        // (the table of contention-free intervals is not in use at this point: it takes every request's longest
        // service time, 4 R bytes, which the host's sweep over the trace needs)
        if (hipGetLastError() != hipSuccess ||
            hipMemcpy(&bounds, d_bounds, sizeof(bounds), hipMemcpyDeviceToHost) != hipSuccess ||
            hipMemcpy(worst_service.data(), w->d_span, 4u * (size_t)w->R, hipMemcpyDeviceToHost) != hipSuccess) {
            (void)hipGetLastError();
            return device_error();
        }
        if (bounds.over_range != 0u || bounds.service_sum > limit - latest) return AP_ERR_RANGE;
        service_sum = bounds.service_sum;
        total += bounds.service_sum;
        latest_unqueued = bounds.latest_unqueued;
        longest_pair = bounds.longest_pair;
        table_longest_prefill = bounds.longest_prefill;
        table_longest_tpot = bounds.longest_tpot;
        for (size_t ki = 0; ki < kinds.size(); ++ki) {      // only a guess is made from these: the kinds are not told apart
            kind_sum[ki] = bounds.service_sum;
            for (uint32_t r = 0; r < w->R; ++r) kind_longest[ki] = std::max<uint64_t>(kind_longest[ki], worst_service[r]);
        }
    }
    for (uint32_t r = 0; r < (on_device ? 0u : w->R); ++r) {
        const uint64_t outl = (uint64_t)w->h_out[r];
        uint64_t worst = 0;
        for (size_t ki = 0; ki < kinds.size(); ++ki) {
            uint64_t prefill, tpot;
            host_cost(kinds[ki], r, prefill, tpot);
            if (tpot > limit || prefill > limit) return AP_ERR_RANGE;
            if (tabled) {
                table_longest_prefill = std::max(table_longest_prefill, prefill);
                table_longest_tpot = std::max(table_longest_tpot, tpot);
            }
            uint64_t svc = prefill + outl * tpot;
            worst = std::max(worst, svc);
            kind_sum[ki] += std::min(svc, limit);
            kind_longest[ki] = std::max(kind_longest[ki], std::min(svc, limit));
        }
        worst_service[r] = (uint32_t)std::min(worst, limit);
        total += worst;
        service_sum += worst;
        latest_unqueued = std::max<uint64_t>(latest_unqueued, (uint64_t)w->h_arrival[r] + worst);
        longest_pair = std::max<uint64_t>(longest_pair, (uint64_t)w->h_arrival[r] + worst - w->h_arrival[r & ~1u]);
        if (total > limit) return AP_ERR_RANGE;
    }

    // ---- LDS plan: the largest chunk that fits ------------------------------------------
    if (hipSetDevice(w->device) != hipSuccess) return device_error();
    int lds_cap = 0, n_cu = 0;
    if (hipDeviceGetAttribute(&lds_cap, hipDeviceAttributeMaxSharedMemoryPerBlock, w->device) != hipSuccess ||
        hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, w->device) != hipSuccess)
        return device_error();
    EvalParams p{};
    p.M = M;
    p.B = B;
    // No bin can count more than R requests, so below 65536 requests two bins share a word.
    const bool hist16 = w->R < 65536u;
    // A chunk should hand each replica about 56 requests, so that the 64-lane blocks of the
    // replay are mostly full and rarely spill into a second block; more than that only costs
    // LDS.  Prefer a size that lets two workgroups share a compute unit (they cover each
    // other's barriers); otherwise take the largest chunk one workgroup can hold.
    const uint32_t want = std::min(kMaxChunk, std::max(2u * kThreads, align_up(56u * M, kThreads)));
    uint32_t bytes = 0, chunk = 0;
    {   // what the kernel itself declares (nothing today) comes off the dynamic part
        hipFuncAttributes attr;
        if (hipFuncGetAttributes(&attr, reinterpret_cast<const void*>(eval_kernel(hist16, w->len16, tabled))) != hipSuccess)
            return device_error();
        lds_cap -= (int)std::min<size_t>(attr.sharedSizeBytes, (size_t)lds_cap);
    }
    for (uint32_t budget : {(uint32_t)lds_cap / 2u, (uint32_t)lds_cap}) {
        const uint32_t smallest = budget == (uint32_t)lds_cap ? kThreads : std::max(kThreads, want / 2u);
        for (chunk = want; chunk >= smallest; chunk -= kThreads) {
            bytes = plan_lds(p, chunk, hist16, w->len16);
            if (bytes <= budget) break;
        }
        if (chunk >= smallest) break;
        chunk = 0;
    }
    // When even the smallest chunk does not fit (large M * B), candidates are scored by the
    // three-kernel pipeline instead, whose slot state is per queue rather than per candidate.
    const bool use_pipeline = chunk == 0;
    if (use_pipeline) bytes = 0;

    // LDS of the kernels that only need the histograms and the accumulators behind them
    const uint32_t hist_bytes = 3u * kBins * (hist16 ? 2u : 4u);
    const uint32_t reduce_lds = hist_bytes + 64u + 3u * kWaves * 4u;

    std::vector<DevReplica> dev(M);
    for (uint32_t m = 0; m < M; ++m) {
        const ap_replica& rp = replicas[m];
        DevReplica& d = dev[m];
        d.a = tabled ? rep_type[m] * w->R : rp.prefill_base_us;     // T * R < 2^32 was checked by the caller
        d.b = tabled ? 0u : rp.prefill_per_tok_us;
        d.c = tabled ? 0u : rp.decode_base_us;
        d.d = tabled ? 0u : rp.decode_per_kctx_us;
        if (rp.t_on_us >= rp.t_off_us || rp.t_off_us <= w->base_us) {
            d.t_on = 0;      // the window is empty or closed before the trace: nothing is ever served
            d.t_off = 0;
        } else {
            d.t_on = rp.t_on_us <= w->base_us ? 0u : (uint32_t)(rp.t_on_us - w->base_us);
            d.t_off = (uint32_t)std::min<uint64_t>(rp.t_off_us - w->base_us, kNever);
        }
    }
    if (tabled) {
        const size_t entries = (size_t)T * w->R;
        if (entries > w->tab_entries && !on_device) {
            if ((w->d_tab_prefill && hipFree(w->d_tab_prefill) != hipSuccess) ||
                (w->d_tab_tpot && hipFree(w->d_tab_tpot) != hipSuccess))
                return device_error();
            w->d_tab_prefill = w->d_tab_tpot = nullptr;
            w->tab_entries = 0;
            w->has_model = false;     // the previous model may have pointed at the freed tables
            if (hipMalloc(&w->d_tab_prefill, entries * 4u) != hipSuccess || hipMalloc(&w->d_tab_tpot, entries * 4u) != hipSuccess) {
                (void)hipGetLastError();
                return AP_ERR_ALLOC;
            }
            w->tab_entries = entries;
        }
        if (on_device && entries > w->tab_entries) return AP_ERR_STATE;       // the caller filled them: they exist
        if (!on_device &&
            (hipMemcpy(w->d_tab_prefill, tab_prefill, entries * 4u, hipMemcpyHostToDevice) != hipSuccess ||
             hipMemcpy(w->d_tab_tpot, tab_tpot, entries * 4u, hipMemcpyHostToDevice) != hipSuccess)) {
            (void)hipGetLastError();
            w->has_model = false;
            return device_error();
        }
    }
    if (hipMemcpy(w->d_rep, dev.data(), sizeof(DevReplica) * M, hipMemcpyHostToDevice) != hipSuccess ||
        (!use_pipeline && hipFuncSetAttribute(reinterpret_cast<const void*>(eval_kernel(hist16, w->len16, tabled)),
                                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess) ||
        hipFuncSetAttribute(hist16 ? reinterpret_cast<const void*>(&k_nominal_metrics<true>)
                                   : reinterpret_cast<const void*>(&k_nominal_metrics<false>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)reduce_lds) != hipSuccess) {
        (void)hipGetLastError();
        w->has_model = false;     // the replica table on the device may be half-written
        return device_error();
    }

    p.arrival = w->d_arrival;
    p.prompt = w->d_prompt;
    p.outlen = w->d_out;
    p.rep = w->d_rep;
    p.tab_prefill = tabled ? w->d_tab_prefill : nullptr;
    p.tab_tpot = tabled ? w->d_tab_tpot : nullptr;
    p.R = w->R;
    p.key_bits = 0;
    while (((M - 1u) >> p.key_bits) != 0u) ++p.key_bits;       // bits needed for the replica ids 0..M-1
    p.slo_ttft = (uint32_t)std::min<uint64_t>(slo->ttft_us, kNever);
    p.slo_tpot = (uint32_t)std::min<uint64_t>(slo->tpot_us, kNever);
    p.penalty = slo->penalty_us;
    p.penalty_bin = ap_hist_bin(slo->penalty_us);
    p.k99 = (uint32_t)((99ull * w->R + 99ull) / 100ull);
    p.replayed = w->d_pending + 2;
    if (hipMemset(p.replayed, 0, sizeof(uint32_t)) != hipSuccess) return device_error();
    w->n_scored = 0;
    w->has_model = false;
    w->has_parent = false;    // its analysis belonged to the previous cost model
    w->tabled = tabled;
    w->params = p;
    w->lds_bytes = bytes;
    w->hist16 = hist16;
    w->n_cu = (uint32_t)n_cu;
    w->max_grid = (uint32_t)n_cu * 64u;    // few candidates per workgroup: the hardware balances uneven finish times
    w->resident_grid = (uint32_t)n_cu * std::max(1u, std::min(4u, bytes ? (uint32_t)lds_cap / bytes : 1u));

    // ---- three-kernel replay: scratch for one batch of candidates -------------------------
    w->reduce_eval = p;
    w->reduce_eval.off_misc = hist_bytes;                              // histograms, then the accumulators
    w->reduce_lds_bytes = reduce_lds;
    w->pipeline = use_pipeline;
    if (use_pipeline) {
        const uint32_t R = w->R;
        const uint32_t chunk_g = std::min(kGroupThreads * kGroupMaxPerThread, align_up(R, kGroupThreads));
        const uint32_t n_chunks = (R + chunk_g - 1u) / chunk_g;
        const uint32_t qs_stride = align_up(M + 2u, 8u);
        const size_t slots = (size_t)n_chunks * chunk_g;               // list positions per candidate
        const size_t per_cand = (size_t)n_chunks * qs_stride * 2u + slots * (2u + 4u + 2u) + (size_t)M * sizeof(QueuePartial) + 4u;
        const size_t target = (size_t)1 << 30;                         // enough candidates per batch to fill the GPU
        uint32_t batch = (uint32_t)std::min<size_t>(65535u, std::max<size_t>(1u, target / per_cand));
        auto carve = [](size_t& off, size_t bytes) { const size_t at = off; off = (off + bytes + 255u) / 256u * 256u; return at; };
        size_t off = 0;
        const size_t o_qs = carve(off, (size_t)batch * n_chunks * qs_stride * 2u);
        const size_t o_list = carve(off, (size_t)batch * slots * 2u);
        const size_t o_te = carve(off, (size_t)batch * slots * 4u);
        const size_t o_p = carve(off, (size_t)batch * slots * 2u);
        const size_t o_part = carve(off, (size_t)batch * M * sizeof(QueuePartial));
        const size_t o_unk = carve(off, (size_t)batch * 4u);
        if (off > w->scratch_bytes) {
            if (w->d_scratch && hipFree(w->d_scratch) != hipSuccess) return device_error();
            w->d_scratch = nullptr;
            w->scratch_bytes = 0;
            if (hipMalloc(&w->d_scratch, off) != hipSuccess) {
                (void)hipGetLastError();
                return AP_ERR_ALLOC;
            }
            w->scratch_bytes = off;
        }
        if (hipMemset(w->d_scratch + o_unk, 0, (size_t)batch * 4u) != hipSuccess) return device_error();
        w->batch = batch;
        GroupParams gp{};
        gp.R = R; gp.M = M; gp.chunk = chunk_g; gp.n_chunks = n_chunks; gp.key_bits = p.key_bits; gp.qs_stride = qs_stride;
        gp.qs = reinterpret_cast<uint16_t*>(w->d_scratch + o_qs);
        gp.list = reinterpret_cast<uint16_t*>(w->d_scratch + o_list);
        gp.unknown = reinterpret_cast<uint32_t*>(w->d_scratch + o_unk);
        gp.replayed = p.replayed;
        w->group_params = gp;
        w->group_lds_bytes = (kGroupWaves * (M + 1u) + M + 2u) * 4u;
        ReplayParams qp{};
        qp.req = w->d_req; qp.rep = w->d_rep; qp.qs = gp.qs; qp.list = gp.list;
        qp.tab_prefill = p.tab_prefill; qp.tab_tpot = p.tab_tpot;
        qp.bins_te = reinterpret_cast<uint32_t*>(w->d_scratch + o_te);
        qp.bins_p = reinterpret_cast<uint16_t*>(w->d_scratch + o_p);
        qp.partial = reinterpret_cast<QueuePartial*>(w->d_scratch + o_part);
        qp.R = R; qp.M = M; qp.B = B; qp.chunk = chunk_g; qp.n_chunks = n_chunks; qp.qs_stride = qs_stride;
        qp.slo_ttft = p.slo_ttft; qp.slo_tpot = p.slo_tpot;
        w->replay_params = qp;
        w->replay_lds_bytes = kReplayWaves * B * kWave * 4u;
        ReduceParams rd{};
        rd.qs = gp.qs; rd.bins_te = qp.bins_te; rd.bins_p = qp.bins_p; rd.partial = qp.partial; rd.unknown = gp.unknown;
        rd.M = M; rd.chunk = chunk_g; rd.n_chunks = n_chunks; rd.qs_stride = qs_stride;
        w->reduce_params = rd;
        if (hipFuncSetAttribute(hist16 ? reinterpret_cast<const void*>(&k_reduce_candidates<true>)
                                       : reinterpret_cast<const void*>(&k_reduce_candidates<false>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)w->reduce_lds_bytes) != hipSuccess)
            return device_error();
    }

    // ---- screening plan: only for identical replicas that are available throughout ------
    bool always_on = true;
    for (const DevReplica& d : dev) always_on = always_on && d.t_on == 0u && d.t_off == kNever;
    w->screen = always_on && kinds.size() == 1 && w->R <= (1u << 30);      // the kernels' byte offsets are 32-bit
    // Screening proves that nobody waits; where the mean number of requests in service per replica (total service time
    // over the trace's span, by Little's law) is a quarter of the slots or more, hardly any candidate will pass, and
    // the trace goes straight to the listed evaluation, which replays every queue.
    const bool crowded = w->span_us == 0 || (double)service_sum / (double)w->span_us / M >= 0.25 * B;
    if (w->screen && crowded && w->d_req8) w->screen = false;
    // The one-wavefront screening kernel hands a step's 64 requests to rings of S slots in no particular order: with
    // few replicas and few slots (64 / M requests per ring and step against S slots) a ring wraps within one step
    // and hardly any candidate passes.  Such tables go to the listed evaluation as well.
    {
        const uint32_t want = std::min(B, kScreenMaxSlots);
        uint32_t S_log2 = 0;
        while ((2u << S_log2) <= want && (M + 1u) * ((2u << S_log2) + 1u) * 4u <= kScreenLdsPerWave) ++S_log2;
        const bool wide = (1u << S_log2) < std::min(want, kScreenMinSlots);
        if (w->screen && !wide && 128u >= M * (1u << S_log2) && w->d_req8) w->screen = false;
    }
    if (w->screen) {
        ScreenParams sp{};
        sp.span = w->d_span;
        sp.span_t = w->d_span_t;
        sp.pair = w->d_pair;
        // the smallest tick that brings every contention-free finish time below 2^16 ticks
        uint64_t tick_us = std::max<uint64_t>(1u, latest_unqueued / 0xFFFDu);
        while (latest_unqueued / tick_us + 2u > 0xFFFFu) ++tick_us;
        sp.nominal = w->d_nominal;
        sp.R = w->R;
        sp.M = M;
        // Screening slots per replica: a power of two, at most B.  One wavefront per candidate as
        // long as that wavefront's slot state (rings and counters of M + 1 replicas) stays small
        // enough for many wavefronts per compute unit with a useful number of slots; otherwise
        // the eight-wavefront kernel, whose workgroup holds one candidate's rings.
        const uint32_t want = std::min(B, kScreenMaxSlots);
        uint32_t S_log2 = 0;
        while ((2u << S_log2) <= want && (M + 1u) * ((2u << S_log2) + 1u) * 4u <= kScreenLdsPerWave) ++S_log2;
        w->screen_wide = (1u << S_log2) < std::min(want, kScreenMinSlots);
        if (w->screen_wide) {
            S_log2 = 0;
            while ((2u << S_log2) <= std::min(B, kWideMaxSlots) && M * (2u << S_log2) * 4u <= kWideLdsBytes) ++S_log2;
        }
        // The eight-wavefront kernel can read one word per pair of requests if the tick is coarse
        // enough for the pair's two tick counts to fit 8 bits (count <= longest_pair / tick + 2).
        // Take that tick when it is not out of proportion: at most twice the other one, or at
        // most an eighth of the mean service time.
        const uint64_t tick_packed = std::max<uint64_t>(tick_us, (longest_pair + 252u) / 253u);
        w->screen_packed = w->screen_wide &&
                           (tick_packed <= 2u * tick_us || tick_packed * 8u <= service_sum / w->R);
        if (w->screen_packed) tick_us = tick_packed;
        sp.slots_log2 = S_log2;
        const uint32_t ring_bytes = 4u << S_log2;
        sp.wave_bytes = ((M + 1u) * (ring_bytes + 4u) + ring_bytes - 1u) / ring_bytes * ring_bytes;
        w->screen_params = sp;
        w->screen_wide_lds_bytes = (((M + 1u) << S_log2) + 4u) * 4u;
        w->screen_lds_bytes = kScreenWaves * sp.wave_bytes;
        // a thread takes two requests per turn; enough workgroups for four turns each, at most one per compute unit
        const uint32_t n_groups = std::max(1u, std::min((uint32_t)n_cu, (w->R + 8u * kThreads - 1u) / (8u * kThreads)));
        if (hipMemsetAsync(w->d_nominal_sums, 0, kNominalSumsBytes, nullptr) != hipSuccess) return device_error();
        hipLaunchKernelGGL(hist16 ? k_nominal_metrics<true> : k_nominal_metrics<false>, dim3(n_groups), dim3(kThreads),
                           reduce_lds, nullptr, w->reduce_eval, w->d_span, w->d_span_t,
                           w->screen_packed ? w->d_pair : nullptr, (uint32_t)tick_us,
                           reinterpret_cast<uint32_t*>(w->d_nominal_sums),
                           reinterpret_cast<unsigned long long*>(w->d_nominal_sums + 3u * kBins * sizeof(uint32_t)), w->d_nominal);
        if (hipGetLastError() != hipSuccess || hipDeviceSynchronize() != hipSuccess) {
            (void)hipGetLastError();
            return device_error();
        }
    }
    // ---- split evaluation: replicas that differ or have windows ---------------------------
    w->split = false;
    if (!w->screen) {
        const ap_status st = plan_split(w, dev, replicas, kinds, worst_service, kind_sum, kind_longest, total,
                                        tabled ? rep_type : nullptr, table_longest_prefill, table_longest_tpot);
        if (st != AP_OK) return st;
    }
    w->has_model = true;
    return AP_OK;
}

ap_status ap_costmodel_set(ap_workload* w, const ap_replica* replicas, uint32_t M, uint32_t B, const ap_slo* slo) {
    return set_cost_model(w, replicas, M, B, slo, nullptr, nullptr, nullptr, 0u);
}

ap_status ap_costtable_set(ap_workload* w, const ap_typed_replica* replicas, uint32_t M, uint32_t B, const ap_slo* slo,
                           const uint32_t* prefill_us, const uint32_t* tpot_us, uint32_t n_types) {
    if (!w || !replicas || !slo || !prefill_us || !tpot_us || M == 0 || B == 0 || n_types == 0) return AP_ERR_INVALID;
    if (M > AP_MAX_REPLICAS) return AP_ERR_RANGE;
    if ((uint64_t)n_types * w->R > 0xFFFFFFFFull) return AP_ERR_RANGE;      // table offsets are 32-bit on the device
    std::vector<ap_replica> plain;
    std::vector<uint32_t> types;
    try {
        plain.resize(M);
        types.resize(M);
    } catch (const std::bad_alloc&) {
        return AP_ERR_ALLOC;
    }
    for (uint32_t m = 0; m < M; ++m) {
        if (replicas[m].type >= n_types) return AP_ERR_INVALID;
        types[m] = replicas[m].type;
        plain[m] = ap_replica{0u, 0u, 0u, 0u, replicas[m].t_on_us, replicas[m].t_off_us};
    }
    return set_cost_model(w, plain.data(), M, B, slo, types.data(), prefill_us, tpot_us, n_types);
}

ap_status ap_eval_candidates(const ap_workload* w, const uint16_t* d_assign, uint32_t C, ap_metrics* d_out,
                             void* hip_stream) {
    if (!w) return AP_ERR_INVALID;
    if (!w->has_model) return AP_ERR_STATE;
    if (C == 0) return AP_OK;
    if (!d_assign || !d_out) return AP_ERR_INVALID;
    w->n_scored += C;
    return launch_dense(w, d_assign, C, d_out, static_cast<hipStream_t>(hip_stream), false, take_pending_word(w));
}

ap_status ap_eval_counts_get(const ap_workload* w, ap_eval_counts* out) {
    if (!w || !out) return AP_ERR_INVALID;
    if (!w->has_model) return AP_ERR_STATE;
    uint32_t replayed = 0;
    if (hipSetDevice(w->device) != hipSuccess || hipDeviceSynchronize() != hipSuccess ||
        hipMemcpy(&replayed, w->d_pending + 2, sizeof(uint32_t), hipMemcpyDeviceToHost) != hipSuccess) {
        (void)hipGetLastError();
        return device_error();
    }
    out->candidates = w->n_scored;
    out->replayed = replayed;
    return AP_OK;
}

ap_status ap_parent_set(ap_workload* w, const uint16_t* parent, uint32_t max_children) {
    if (!w || !parent || max_children == 0) return AP_ERR_INVALID;
    if (!w->has_model) return AP_ERR_STATE;
    if (hipSetDevice(w->device) != hipSuccess) return device_error();
    w->has_parent = false;
    if ((uint64_t)max_children > (UINT64_MAX / sizeof(uint16_t)) / w->R) return AP_ERR_ALLOC;     // the rows cannot exist
    const size_t need = (size_t)max_children * w->R * sizeof(uint16_t);
    const size_t row_bytes = (size_t)w->R * sizeof(uint16_t), peak_bytes = sizeof(uint32_t) * (AP_MAX_REPLICAS + 1u);
    if ((!w->d_parent && hipMalloc(&w->d_parent, row_bytes) != hipSuccess) ||
        (!w->d_peak && hipMalloc(&w->d_peak, peak_bytes) != hipSuccess) ||
        (!w->d_room && hipMalloc(&w->d_room, sizeof(uint32_t) * AP_MAX_REPLICAS) != hipSuccess) ||
        (!w->h_stage && hipHostMalloc(reinterpret_cast<void**>(&w->h_stage), std::max(row_bytes, peak_bytes), hipHostMallocDefault) != hipSuccess)) {
        (void)hipGetLastError();
        return AP_ERR_ALLOC;
    }
    if (need > w->rows_bytes) {
        if (w->d_rows && hipFree(w->d_rows) != hipSuccess) return device_error();
        w->d_rows = nullptr;
        w->rows_bytes = 0;
        if (hipMalloc(&w->d_rows, need) != hipSuccess) {
            (void)hipGetLastError();
            return AP_ERR_ALLOC;
        }
        w->rows_bytes = need;
    }
    // through the pinned buffer: upload, analysis and read-back are queued together and waited for once
    std::memcpy(w->h_stage, parent, row_bytes);
    if (hipMemcpyAsync(w->d_parent, w->h_stage, row_bytes, hipMemcpyHostToDevice, nullptr) != hipSuccess) return device_error();
    const uint32_t M = w->params.M;
    bool certify = false;
    if (w->screen) {
        // the shortcut needs the nominal record, i.e. identical replicas that are always available
        hipLaunchKernelGGL(k_parent_occupancy, dim3(M), dim3(kOccupancyThreads), 0, nullptr, w->params, w->d_parent, w->d_peak,
                           w->d_room);
        // (the kernel is queued behind the upload, which has therefore read the pinned buffer before the depths land in it)
        if (hipGetLastError() != hipSuccess ||
            hipMemcpyAsync(w->h_stage, w->d_peak, sizeof(uint32_t) * (M + 1u), hipMemcpyDeviceToHost, nullptr) != hipSuccess ||
            hipStreamSynchronize(nullptr) != hipSuccess) {
            (void)hipGetLastError();
            return device_error();
        }
        const uint32_t* peak = reinterpret_cast<const uint32_t*>(w->h_stage);
        // ... and a parent that is contention-free itself and names only replicas of the table
        certify = peak[M] == 0u;
        for (uint32_t m = 0; m < M; ++m) certify = certify && peak[m] <= w->params.B;
    } else if (hipStreamSynchronize(nullptr) != hipSuccess) {
        (void)hipGetLastError();
        return device_error();
    }
    ChildParams cp{};
    cp.parent = w->d_parent;
    cp.room = w->d_room;
    cp.nominal = w->d_nominal;
    cp.rows = w->d_rows;
    cp.R = w->R;
    cp.M = M;
    cp.key_bits = 0;
    while (((w->R - 1u) >> cp.key_bits) != 0u) ++cp.key_bits;
    cp.certify = certify ? 1u : 0u;
    w->child_params = cp;
    w->max_children = max_children;
    w->has_parent = true;
    return AP_OK;
}

ap_status ap_eval_children(const ap_workload* w, const uint32_t* d_edit_first, const uint32_t* d_edit_request,
                           const uint16_t* d_edit_replica, uint32_t C, ap_metrics* d_out, void* hip_stream) {
    if (!w) return AP_ERR_INVALID;
    if (!w->has_model || !w->has_parent) return AP_ERR_STATE;
    if (C == 0) return AP_OK;
    if (!d_edit_first || !d_edit_request || !d_edit_replica || !d_out) return AP_ERR_INVALID;
    if (C > w->max_children) return AP_ERR_RANGE;
    w->n_scored += C;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const uint32_t blocks = std::min((C + kChildWaves - 1u) / kChildWaves, w->n_cu * 64u);
    const PendingWord flags = take_pending_word(w);
    hipLaunchKernelGGL(k_certify_children, dim3(blocks), dim3(kChildThreads), (kChildWaves + 1u) * w->child_params.M * 4u, stream,
                       w->child_params, d_edit_first, d_edit_request, d_edit_replica, d_out, C, flags);
    if (hipGetLastError() != hipSuccess) return device_error();
    return launch_dense(w, w->d_rows, C, d_out, stream, w->child_params.certify != 0u, flags);
}

// ---- roofline cost tables -------------------------------------------------------------
namespace {

// Validate the descriptions and run the table kernels; leaves prefill_ns / prefix_ns / weight_bytes /
// feasible filled on the device.
ap_status roofline_tables_on_device(const ap_model* models, uint32_t n_models, const ap_gpu* gpus, uint32_t n_gpus,
                                    const ap_group* groups, uint32_t n_groups, uint32_t max_seq, RoofBuffers& buf) {
    if (!models || !gpus || !groups || n_models == 0 || n_gpus == 0 || n_groups == 0 || max_seq == 0) return AP_ERR_INVALID;
    if (n_groups > 65535u || max_seq > (1u << 24)) return AP_ERR_RANGE;
    std::vector<RoofGroup> host;
    try {
        host.resize(n_groups);
    } catch (const std::bad_alloc&) {
        return AP_ERR_ALLOC;
    }
    for (uint32_t i = 0; i < n_groups; ++i) {
        const ap_group& gr = groups[i];
        if (gr.model >= n_models || gr.gpu >= n_gpus || gr.tp == 0 || gr.batch == 0) return AP_ERR_INVALID;
        const ap_model& m = models[gr.model];
        const ap_gpu& g = gpus[gr.gpu];
        if (m.layers == 0 || m.hidden == 0 || m.intermediate == 0 || m.vocab == 0 || m.heads == 0 || m.kv_heads == 0 ||
            m.kv_heads > m.heads || m.weight_bits == 0)
            return AP_ERR_INVALID;
        if (!(g.flops > 0.0) || !(g.hbm_bytes_per_s > 0.0) || !(g.mem_bytes > 0.0) || g.gpus_per_node == 0 ||
            !(g.link_intra_bytes_per_s > 0.0) || !(g.link_inter_bytes_per_s > 0.0))
            return AP_ERR_INVALID;
        RoofGroup& o = host[i];
        o.L = m.layers; o.H = m.hidden; o.I = m.intermediate; o.V = m.vocab; o.A = m.heads; o.K = m.kv_heads;
        o.e = (double)m.weight_bits / 8.0;
        o.b = gr.batch; o.t = gr.tp;
        o.flops = g.flops; o.hbm = g.hbm_bytes_per_s;
        o.link = gr.tp <= g.gpus_per_node ? g.link_intra_bytes_per_s : g.link_inter_bytes_per_s;
        o.mem = g.mem_bytes;
    }
    const size_t per_group = (size_t)max_seq + 1u;
    if (n_groups > buf.cap_groups || max_seq > buf.cap_seq) {
        buf.release();
        if (hipMalloc(&buf.groups, sizeof(RoofGroup) * n_groups) != hipSuccess ||
            hipMalloc(&buf.prefill_ns, 8u * per_group * n_groups) != hipSuccess ||
            hipMalloc(&buf.step_ns, 8u * per_group * n_groups) != hipSuccess ||
            hipMalloc(&buf.prefix_ns, 8u * (per_group + 1u) * n_groups) != hipSuccess ||
            hipMalloc(&buf.weight_bytes, 8u * n_groups) != hipSuccess || hipMalloc(&buf.feasible, 4u * n_groups) != hipSuccess) {
            (void)hipGetLastError();
            buf.release();
            return AP_ERR_ALLOC;
        }
        buf.cap_groups = n_groups;
        buf.cap_seq = max_seq;
    }
    if (hipMemcpy(buf.groups, host.data(), sizeof(RoofGroup) * n_groups, hipMemcpyHostToDevice) != hipSuccess) {
        (void)hipGetLastError();
        return device_error();
    }
    hipLaunchKernelGGL(k_roofline_steps, dim3((max_seq + kRoofThreads) / kRoofThreads, n_groups), dim3(kRoofThreads), 0, nullptr,
                       buf.groups, n_groups, max_seq, buf.prefill_ns, buf.step_ns, buf.weight_bytes, buf.feasible);
    hipLaunchKernelGGL(k_roofline_prefix, dim3(n_groups), dim3(kRoofThreads), 0, nullptr, buf.step_ns, max_seq, buf.prefix_ns);
    if (hipGetLastError() != hipSuccess) return device_error();
    return AP_OK;
}

}  // namespace

ap_status ap_costtable_set_roofline(ap_workload* w, const ap_typed_replica* replicas, uint32_t M, uint32_t B,
                                    const ap_slo* slo, const ap_model* models, uint32_t n_models, const ap_gpu* gpus,
                                    uint32_t n_gpus, const ap_group* groups, uint32_t n_groups) {
    if (!w || !replicas || !slo || M == 0 || B == 0 || n_groups == 0) return AP_ERR_INVALID;
    if (M > AP_MAX_REPLICAS) return AP_ERR_RANGE;
    if ((uint64_t)n_groups * w->R > 0xFFFFFFFFull) return AP_ERR_RANGE;     // table offsets are 32-bit on the device
    if (hipSetDevice(w->device) != hipSuccess) return device_error();
    std::vector<ap_replica> plain;
    std::vector<uint32_t> types;
    try {
        plain.resize(M);
        types.resize(M);
        if (!w->roof) w->roof = new RoofBuffers;
    } catch (const std::bad_alloc&) {
        return AP_ERR_ALLOC;
    }
    for (uint32_t m = 0; m < M; ++m) {
        if (replicas[m].type >= n_groups) return AP_ERR_INVALID;
        types[m] = replicas[m].type;
        plain[m] = ap_replica{0u, 0u, 0u, 0u, replicas[m].t_on_us, replicas[m].t_off_us};
    }
    uint64_t longest = 0;                                  // prompt + output of the longest request
    for (uint32_t r = 0; r < w->R; ++r) longest = std::max<uint64_t>(longest, (uint64_t)w->h_prompt[r] + (uint64_t)w->h_out[r]);
    if (longest > (1u << 24)) return AP_ERR_RANGE;
    const ap_status st = roofline_tables_on_device(models, n_models, gpus, n_gpus, groups, n_groups, (uint32_t)longest, *w->roof);
    if (st != AP_OK) return st;
    // from here on the previous cost model is gone: the tables it may have read are overwritten
    w->has_model = false;
    const size_t entries = (size_t)n_groups * w->R;
    if (entries > w->tab_entries) {
        if ((w->d_tab_prefill && hipFree(w->d_tab_prefill) != hipSuccess) || (w->d_tab_tpot && hipFree(w->d_tab_tpot) != hipSuccess)) {
            (void)hipGetLastError();
            return device_error();
        }
        w->d_tab_prefill = w->d_tab_tpot = nullptr;
        w->tab_entries = 0;
        if (hipMalloc(&w->d_tab_prefill, entries * 4u) != hipSuccess || hipMalloc(&w->d_tab_tpot, entries * 4u) != hipSuccess) {
            (void)hipGetLastError();
            return AP_ERR_ALLOC;
        }
        w->tab_entries = entries;
    }
    if (!w->d_bounds && hipMalloc(&w->d_bounds, sizeof(TableBounds) + 4u * AP_MAX_REPLICAS) != hipSuccess) {
        (void)hipGetLastError();
        return AP_ERR_ALLOC;
    }
    hipLaunchKernelGGL(k_roofline_request_costs, dim3((w->R + kRoofThreads - 1u) / kRoofThreads, n_groups), dim3(kRoofThreads),
                       0, nullptr, w->roof->prefill_ns, w->roof->prefix_ns, (uint32_t)longest, w->d_prompt, w->d_out, w->R,
                       w->d_tab_prefill, w->d_tab_tpot);
    if (hipGetLastError() != hipSuccess) return device_error();
    return set_cost_model(w, plain.data(), M, B, slo, types.data(), nullptr, nullptr, n_groups);
}

ap_status ap_roofline_tables(const ap_model* models, uint32_t n_models, const ap_gpu* gpus, uint32_t n_gpus,
                             const ap_group* groups, uint32_t n_groups, uint32_t max_seq, uint64_t* prefill_ns,
                             uint64_t* decode_prefix_ns, double* weight_bytes, uint8_t* feasible) {
    if (!prefill_ns || !decode_prefix_ns || !weight_bytes || !feasible) return AP_ERR_INVALID;
    RoofBuffers buf;
    const ap_status st = roofline_tables_on_device(models, n_models, gpus, n_gpus, groups, n_groups, max_seq, buf);
    if (st != AP_OK) return st;
    std::vector<uint32_t> ok;
    try {
        ok.resize(n_groups);
    } catch (const std::bad_alloc&) {
        return AP_ERR_ALLOC;
    }
    const size_t per_group = (size_t)max_seq + 1u;
    if (hipMemcpy(prefill_ns, buf.prefill_ns, 8u * per_group * n_groups, hipMemcpyDeviceToHost) != hipSuccess ||
        hipMemcpy(decode_prefix_ns, buf.prefix_ns, 8u * (per_group + 1u) * n_groups, hipMemcpyDeviceToHost) != hipSuccess ||
        hipMemcpy(weight_bytes, buf.weight_bytes, 8u * n_groups, hipMemcpyDeviceToHost) != hipSuccess ||
        hipMemcpy(ok.data(), buf.feasible, 4u * n_groups, hipMemcpyDeviceToHost) != hipSuccess) {
        (void)hipGetLastError();
        return device_error();
    }
    for (uint32_t i = 0; i < n_groups; ++i) feasible[i] = ok[i] ? 1u : 0u;
    return AP_OK;
}

ap_status ap_roofline_costs(const ap_workload* w, const ap_model* models, uint32_t n_models, const ap_gpu* gpus,
                            uint32_t n_gpus, const ap_group* groups, uint32_t n_groups, uint32_t* prefill_us,
                            uint32_t* tpot_us) {
    if (!w || !prefill_us || !tpot_us) return AP_ERR_INVALID;
    if (hipSetDevice(w->device) != hipSuccess) return device_error();
    uint64_t longest = 0;                                  // prompt + output of the longest request
    for (uint32_t r = 0; r < w->R; ++r) longest = std::max<uint64_t>(longest, (uint64_t)w->h_prompt[r] + (uint64_t)w->h_out[r]);
    if (longest > (1u << 24)) return AP_ERR_RANGE;
    RoofBuffers buf;
    const ap_status st = roofline_tables_on_device(models, n_models, gpus, n_gpus, groups, n_groups, (uint32_t)longest, buf);
    if (st != AP_OK) return st;
    const size_t entries = (size_t)n_groups * w->R;
    if (hipMalloc(&buf.prefill_us, 4u * entries) != hipSuccess || hipMalloc(&buf.tpot_us, 4u * entries) != hipSuccess) {
        (void)hipGetLastError();
        return AP_ERR_ALLOC;
    }
    hipLaunchKernelGGL(k_roofline_request_costs, dim3((w->R + kRoofThreads - 1u) / kRoofThreads, n_groups), dim3(kRoofThreads),
                       0, nullptr, buf.prefill_ns, buf.prefix_ns, (uint32_t)longest, w->d_prompt, w->d_out, w->R, buf.prefill_us,
                       buf.tpot_us);
    if (hipGetLastError() != hipSuccess ||
        hipMemcpy(prefill_us, buf.prefill_us, 4u * entries, hipMemcpyDeviceToHost) != hipSuccess ||
        hipMemcpy(tpot_us, buf.tpot_us, 4u * entries, hipMemcpyDeviceToHost) != hipSuccess) {
        (void)hipGetLastError();
        return device_error();
    }
    return AP_OK;
}

ap_status ap_trace_time(const ap_model* models, const double* pcie_coef, uint32_t n_models, const ap_gpu* gpus, uint32_t n_gpus,
                        const ap_placement* d_plans, const uint32_t* d_n_intervals, const uint64_t* d_sched_ns,
                        const uint64_t* d_stale_ns, const uint64_t* d_serve_ns, uint32_t C, uint32_t N_max,
                        uint32_t load_scope, ap_breakdown* d_out, void* hip_stream) {
    if (!models || !pcie_coef || !gpus || n_models == 0 || n_gpus == 0 || N_max == 0) return AP_ERR_INVALID;
    if (load_scope != AP_LOAD_DEPLOYED && load_scope != AP_LOAD_CHANGED) return AP_ERR_INVALID;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (C == 0) return AP_OK;
    if (!d_plans || !d_n_intervals || !d_sched_ns || !d_stale_ns || !d_serve_ns || !d_out) return AP_ERR_INVALID;
    if ((uint64_t)n_models * n_gpus > (1u << 20)) return AP_ERR_RANGE;
    std::vector<RoofGroup> host;
    std::vector<double> pcie;
    try {
        host.resize(n_models);
        pcie.resize(n_gpus);
    } catch (const std::bad_alloc&) {
        return AP_ERR_ALLOC;
    }
    for (uint32_t z = 0; z < n_models; ++z) {
        const ap_model& m = models[z];
        if (m.layers == 0 || m.hidden == 0 || m.intermediate == 0 || m.vocab == 0 || m.heads == 0 || m.kv_heads == 0 ||
            m.kv_heads > m.heads || m.weight_bits == 0 || !(pcie_coef[z] > 0.0))
            return AP_ERR_INVALID;
        RoofGroup o{};
        o.L = m.layers; o.H = m.hidden; o.I = m.intermediate; o.V = m.vocab; o.A = m.heads; o.K = m.kv_heads;
        o.e = (double)m.weight_bits / 8.0;
        host[z] = o;
    }
    for (uint32_t g = 0; g < n_gpus; ++g) {
        if (!(gpus[g].pcie_bytes_per_s > 0.0)) return AP_ERR_INVALID;
        pcie[g] = gpus[g].pcie_bytes_per_s;
    }
    struct Temp {
        RoofGroup* models = nullptr;
        double* coef = nullptr;
        double* pcie = nullptr;
        unsigned long long* tau = nullptr;
        ~Temp() {
            for (void* q : {(void*)models, (void*)coef, (void*)pcie, (void*)tau})
                if (q) (void)hipFree(q);
        }
    } tmp;
    if (hipMalloc(&tmp.models, sizeof(RoofGroup) * n_models) != hipSuccess || hipMalloc(&tmp.coef, 8u * n_models) != hipSuccess ||
        hipMalloc(&tmp.pcie, 8u * n_gpus) != hipSuccess || hipMalloc(&tmp.tau, 8u * (size_t)n_models * n_gpus) != hipSuccess) {
        (void)hipGetLastError();
        return AP_ERR_ALLOC;
    }
    // the descriptions are on the device when these copies return; the kernels then run on the caller's stream,
    // behind whatever produced the device inputs there
    if (hipMemcpy(tmp.models, host.data(), sizeof(RoofGroup) * n_models, hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(tmp.coef, pcie_coef, 8u * n_models, hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(tmp.pcie, pcie.data(), 8u * n_gpus, hipMemcpyHostToDevice) != hipSuccess) {
        (void)hipGetLastError();
        return device_error();
    }
    hipLaunchKernelGGL(k_transfer_times, dim3((n_models * n_gpus + kRoofThreads - 1u) / kRoofThreads), dim3(kRoofThreads), 0, stream,
                       tmp.models, tmp.coef, n_models, tmp.pcie, n_gpus, tmp.tau);
    TraceTimeParams tp{};
    tp.tau_ns = tmp.tau;
    tp.plans = d_plans;
    tp.n_intervals = d_n_intervals;
    tp.sched_ns = reinterpret_cast<const unsigned long long*>(d_sched_ns);
    tp.stale_ns = reinterpret_cast<const unsigned long long*>(d_stale_ns);
    tp.serve_ns = reinterpret_cast<const unsigned long long*>(d_serve_ns);
    tp.C = C; tp.N_max = N_max; tp.Z = n_models; tp.G = n_gpus;
    tp.load_changed_only = load_scope == AP_LOAD_CHANGED ? 1u : 0u;
    hipLaunchKernelGGL(k_trace_time, dim3((C + kRoofThreads - 1u) / kRoofThreads), dim3(kRoofThreads), 0, stream, tp, d_out);
    // the temporary tables are freed on return: wait for the stream
    if (hipGetLastError() != hipSuccess || hipStreamSynchronize(stream) != hipSuccess) {
        (void)hipGetLastError();
        return device_error();
    }
    return AP_OK;
}

// ---- trace time for callers that cannot allocate ------------------------------------------
// The transfer-time table of ap_trace_time_static lives in this array (one copy per device, held until the
// process ends).  In host code the array's name is only a stand-in for the symbol: its device address is asked
// for once per device and kept in trace_scratch_at.
static __device__ __align__(256) unsigned long long scratch[kTransferArgModels * kTransferArgGpus];
constexpr int kScratchDevices = 64;
static unsigned long long* trace_scratch_at[kScratchDevices] = {};
static std::mutex trace_scratch_lock;

ap_status ap_trace_time_static(const ap_model* models, const double* pcie_coef, uint32_t n_models, const ap_gpu* gpus,
                               uint32_t n_gpus, const ap_placement* d_plans, const uint32_t* d_n_intervals,
                               const uint64_t* d_sched_ns, const uint64_t* d_stale_ns, const uint64_t* d_serve_ns, uint32_t C,
                               uint32_t N_max, uint32_t load_scope, ap_breakdown* d_out, void* hip_stream) {
    if (!models || !pcie_coef || !gpus || n_models == 0 || n_gpus == 0 || N_max == 0) return AP_ERR_INVALID;
    if (load_scope != AP_LOAD_DEPLOYED && load_scope != AP_LOAD_CHANGED) return AP_ERR_INVALID;
    if (n_models > AP_STATIC_MAX_MODELS || n_gpus > AP_STATIC_MAX_GPU_TYPES) return AP_ERR_RANGE;
    if (C == 0) return AP_OK;
    if (!d_plans || !d_n_intervals || !d_sched_ns || !d_stale_ns || !d_serve_ns || !d_out) return AP_ERR_INVALID;
    TransferArgs args{};
    for (uint32_t z = 0; z < n_models; ++z) {
        const ap_model& m = models[z];
        if (m.layers == 0 || m.hidden == 0 || m.intermediate == 0 || m.vocab == 0 || m.heads == 0 || m.kv_heads == 0 ||
            m.kv_heads > m.heads || m.weight_bits == 0 || !(pcie_coef[z] > 0.0))
            return AP_ERR_INVALID;
        args.model[z] = m;
        args.coef[z] = pcie_coef[z];
    }
    for (uint32_t g = 0; g < n_gpus; ++g) {
        if (!(gpus[g].pcie_bytes_per_s > 0.0)) return AP_ERR_INVALID;
        args.pcie[g] = gpus[g].pcie_bytes_per_s;
    }
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) return device_error();
    if (device < 0 || device >= kScratchDevices) return AP_ERR_RANGE;
    unsigned long long* tau = nullptr;
    {
        std::lock_guard<std::mutex> hold(trace_scratch_lock);
        if (!trace_scratch_at[device]) {                      // the first call on this device, which is current
            void* at = nullptr;
            if (hipGetSymbolAddress(&at, HIP_SYMBOL(scratch)) != hipSuccess || !at) {
                (void)hipGetLastError();
                return device_error();
            }
            trace_scratch_at[device] = static_cast<unsigned long long*>(at);
        }
        tau = trace_scratch_at[device];
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    // every entry the second kernel reads is written by the first: nothing of an earlier call is looked at
    hipLaunchKernelGGL(k_transfer_times_from_args, dim3((n_models * n_gpus + kRoofThreads - 1u) / kRoofThreads), dim3(kRoofThreads), 0,
                       stream, args, n_models, n_gpus, tau);
    TraceTimeParams tp{};
    tp.tau_ns = tau;
    tp.plans = d_plans;
    tp.n_intervals = d_n_intervals;
    tp.sched_ns = reinterpret_cast<const unsigned long long*>(d_sched_ns);
    tp.stale_ns = reinterpret_cast<const unsigned long long*>(d_stale_ns);
    tp.serve_ns = reinterpret_cast<const unsigned long long*>(d_serve_ns);
    tp.C = C; tp.N_max = N_max; tp.Z = n_models; tp.G = n_gpus;
    tp.load_changed_only = load_scope == AP_LOAD_CHANGED ? 1u : 0u;
    hipLaunchKernelGGL(k_trace_time, dim3((C + kRoofThreads - 1u) / kRoofThreads), dim3(kRoofThreads), 0, stream, tp, d_out);
    if (hipGetLastError() != hipSuccess) return device_error();
    return AP_OK;
}

// ---- agentic workflows ------------------------------------------------------------------
struct ap_agentic {
    int device = 0;
    AgenticParams params{};
    uint32_t lds_bytes = 0;
    uint32_t n_cu = 0;
    void* d_block = nullptr;          // one allocation behind all the tables
};

ap_status ap_agentic_create(const uint64_t* arrival_us, const uint64_t* slo_us, uint32_t W, const uint32_t* wf,
                            const uint32_t* in_len, const uint32_t* out_len, const uint32_t* pred_first, const uint32_t* pred,
                            uint32_t K, const ap_prefill_instance* prefill, uint32_t P, const ap_decode_instance* decode,
                            uint32_t Q, uint64_t penalty_permille, ap_agentic** out) {
    if (!arrival_us || !slo_us || !wf || !in_len || !out_len || !pred_first || !prefill || !decode || !out || W == 0 || K == 0 ||
        P == 0 || Q == 0)
        return AP_ERR_INVALID;
    if (W > AP_AGENTIC_MAX_WORKFLOWS || K > AP_AGENTIC_MAX_CALLS || P > AP_AGENTIC_MAX_INSTANCES || Q > AP_AGENTIC_MAX_INSTANCES)
        return AP_ERR_RANGE;
    if (pred_first[0] != 0u) return AP_ERR_INVALID;
    for (uint32_t k = 0; k < K; ++k) {
        if (wf[k] >= W || in_len[k] == 0 || out_len[k] == 0 || pred_first[k + 1u] < pred_first[k]) return AP_ERR_INVALID;
        if (pred_first[k + 1u] > pred_first[k] && !pred) return AP_ERR_INVALID;
        for (uint32_t i = pred_first[k]; i < pred_first[k + 1u]; ++i)
            if (pred[i] >= k || wf[pred[i]] != wf[k]) return AP_ERR_INVALID;
    }
    uint64_t first = arrival_us[0], last = arrival_us[0];
    for (uint32_t w = 0; w < W; ++w) {
        if (slo_us[w] == 0) return AP_ERR_INVALID;
        first = std::min(first, arrival_us[w]);
        last = std::max(last, arrival_us[w]);
    }
    for (uint32_t i = 0; i < P; ++i)
        if ((uint64_t)prefill[i].base_us + prefill[i].per_tok_us == 0) return AP_ERR_INVALID;
    for (uint32_t i = 0; i < Q; ++i)
        if ((uint64_t)decode[i].base_us + decode[i].per_kctx_us == 0) return AP_ERR_INVALID;
    // 32-bit time: no completion can lie beyond the last arrival plus every call's slowest stages in a row
    const uint64_t limit = (uint64_t)kNever - 1u;
    uint64_t total = last - first;
    if (total > limit) return AP_ERR_RANGE;
    for (uint32_t k = 0; k < K; ++k) {
        uint64_t slow_pre = 0, slow_dec = 0;
        for (uint32_t i = 0; i < P; ++i)
            slow_pre = std::max<uint64_t>(slow_pre, (uint64_t)prefill[i].base_us + (uint64_t)prefill[i].per_tok_us * in_len[k]);
        for (uint32_t i = 0; i < Q; ++i)
            slow_dec = std::max<uint64_t>(slow_dec, (uint64_t)out_len[k] * ((uint64_t)decode[i].base_us +
                                                    (uint64_t)decode[i].per_kctx_us * (((uint64_t)in_len[k] + 1023u) >> 10)));
        if (slow_pre > limit || slow_dec > limit) return AP_ERR_RANGE;
        total += slow_pre + slow_dec;
        if (total > limit) return AP_ERR_RANGE;
        if ((uint64_t)in_len[k] + out_len[k] > limit) return AP_ERR_RANGE;
    }

    ap_agentic* a = new (std::nothrow) ap_agentic;
    if (!a) return AP_ERR_ALLOC;
    ap_status st = AP_OK;
    const uint32_t n_pred = pred_first[K];
    std::vector<uint32_t> rel, pa, pb, qc, qd, cap;
    try {
        rel.resize(W); pa.resize(P); pb.resize(P); qc.resize(Q); qd.resize(Q); cap.resize(Q);
    } catch (const std::bad_alloc&) {
        delete a;
        return AP_ERR_ALLOC;
    }
    for (uint32_t w = 0; w < W; ++w) rel[w] = (uint32_t)(arrival_us[w] - first);
    // the kernel counts down a call's outstanding predecessors, so it wants the lists the other way round
    std::vector<uint32_t> n_pred_of, succ_first, succ;
    try {
        n_pred_of.assign(K, 0u);
        succ_first.assign(K + 1u, 0u);
        succ.assign(std::max(1u, n_pred), 0u);
    } catch (const std::bad_alloc&) {
        delete a;
        return AP_ERR_ALLOC;
    }
    try {                                                   // the temporaries below allocate
        for (uint32_t k = 0; k < K; ++k) {
            // a predecessor listed twice counts once: keep distinct ones
            std::vector<uint32_t> mine(pred + pred_first[k], pred + pred_first[k + 1u]);
            std::sort(mine.begin(), mine.end());
            mine.erase(std::unique(mine.begin(), mine.end()), mine.end());
            if (mine.size() > 255u) { delete a; return AP_ERR_RANGE; }
            n_pred_of[k] = (uint32_t)mine.size();
            for (uint32_t j : mine) ++succ_first[j + 1u];
        }
        for (uint32_t k = 0; k < K; ++k) succ_first[k + 1u] += succ_first[k];
        {
            std::vector<uint32_t> fill(succ_first.begin(), succ_first.end() - 1);
            for (uint32_t k = 0; k < K; ++k) {
                std::vector<uint32_t> mine(pred + pred_first[k], pred + pred_first[k + 1u]);
                std::sort(mine.begin(), mine.end());
                mine.erase(std::unique(mine.begin(), mine.end()), mine.end());
                for (uint32_t j : mine) succ[fill[j]++] = k;
            }
        }
    } catch (const std::bad_alloc&) {
        delete a;
        return AP_ERR_ALLOC;
    }
    for (uint32_t i = 0; i < P; ++i) { pa[i] = prefill[i].base_us; pb[i] = prefill[i].per_tok_us; }
    for (uint32_t i = 0; i < Q; ++i) { qc[i] = decode[i].base_us; qd[i] = decode[i].per_kctx_us; cap[i] = decode[i].capacity_tokens; }
    // one block: slo (8-byte entries) first, then the 4-byte tables
    const size_t n_words = (size_t)W + 4u * K + (K + 1u) + std::max(1u, n_pred) + 2u * P + 3u * Q;
    const size_t bytes = 8u * (size_t)W + 4u * n_words;
    if (hipGetDevice(&a->device) != hipSuccess) st = AP_ERR_DEVICE;
    if (st == AP_OK && hipMalloc(&a->d_block, bytes) != hipSuccess) st = AP_ERR_ALLOC;
    int n_cu = 0, lds_cap = 0;
    if (st == AP_OK && (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, a->device) != hipSuccess ||
                        hipDeviceGetAttribute(&lds_cap, hipDeviceAttributeMaxSharedMemoryPerBlock, a->device) != hipSuccess))
        st = AP_ERR_DEVICE;
    if (st == AP_OK) {
        unsigned char* base = static_cast<unsigned char*>(a->d_block);
        unsigned long long* d_slo = reinterpret_cast<unsigned long long*>(base);
        uint32_t* at = reinterpret_cast<uint32_t*>(base + 8u * (size_t)W);
        auto put = [&](const uint32_t* src, size_t n) {
            uint32_t* here = at;
            if (n && hipMemcpy(here, src, 4u * n, hipMemcpyHostToDevice) != hipSuccess) st = AP_ERR_DEVICE;
            at += n;
            return here;
        };
        if (hipMemcpy(d_slo, slo_us, 8u * (size_t)W, hipMemcpyHostToDevice) != hipSuccess) st = AP_ERR_DEVICE;
        AgenticParams& p = a->params;
        p.slo = d_slo;
        p.arrival = put(rel.data(), W);
        p.wf = put(wf, K);
        p.in_len = put(in_len, K);
        p.out_len = put(out_len, K);
        p.n_pred = put(n_pred_of.data(), K);
        p.succ_first = put(succ_first.data(), K + 1u);
        p.succ = put(succ.data(), std::max(1u, n_pred));
        p.pa = put(pa.data(), P);
        p.pb = put(pb.data(), P);
        p.qc = put(qc.data(), Q);
        p.qd = put(qd.data(), Q);
        p.cap = put(cap.data(), Q);
        p.penalty = penalty_permille;
        p.W = W; p.K = K; p.P = P; p.Q = Q;
        // per wavefront: key u32[max(K, 2W)] (later ratio u64[W]) | tev u32[K] | comp u32[W] | used u32[Q] | ids u16[2K] |
        // phase, left u8[K] each | busy u8[P] | failed u8[W]
        const uint32_t wave_bytes = align_up(4u * (std::max(K, 2u * W) + K + W + Q) + 2u * 2u * K + 2u * K + P + W, 16u);
        p.wave_bytes = wave_bytes;
        a->lds_bytes = wave_bytes * kAgenticWaves;
        a->n_cu = (uint32_t)n_cu;
        if (a->lds_bytes > (uint32_t)lds_cap) st = AP_ERR_RANGE;
        else if (hipFuncSetAttribute(reinterpret_cast<const void*>(&k_agentic_eval), hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)a->lds_bytes) != hipSuccess)
            st = AP_ERR_DEVICE;
    }
    if (st != AP_OK) {
        (void)hipGetLastError();
        ap_agentic_destroy(a);
        return st;
    }
    *out = a;
    return AP_OK;
}

ap_status ap_agentic_eval(const ap_agentic* a, const uint16_t* d_prefill, const uint16_t* d_decode, const uint32_t* d_key,
                          uint32_t C, ap_agentic_metrics* d_out, void* hip_stream) {
    if (!a) return AP_ERR_INVALID;
    if (C == 0) return AP_OK;
    if (!d_prefill || !d_decode || !d_key || !d_out) return AP_ERR_INVALID;
    const uint32_t blocks = std::min((C + kAgenticWaves - 1u) / kAgenticWaves, a->n_cu * 64u);
    hipLaunchKernelGGL(k_agentic_eval, dim3(blocks), dim3(kAgenticThreads), a->lds_bytes, static_cast<hipStream_t>(hip_stream),
                       a->params, d_prefill, d_decode, d_key, d_out, C);
    if (hipGetLastError() != hipSuccess) return device_error();
    return AP_OK;
}

ap_status ap_agentic_destroy(ap_agentic* a) {
    if (!a) return AP_OK;
    const bool ok = !a->d_block || hipFree(a->d_block) == hipSuccess;
    delete a;
    return ok ? AP_OK : AP_ERR_DEVICE;
}

ap_status ap_workload_destroy(ap_workload* w) {
    if (!w) return AP_OK;
    bool ok = true;
    if (w->d_arrival) ok = (hipFree(w->d_arrival) == hipSuccess) && ok;
    if (w->d_prompt) ok = (hipFree(w->d_prompt) == hipSuccess) && ok;
    if (w->d_out) ok = (hipFree(w->d_out) == hipSuccess) && ok;
    if (w->d_rep) ok = (hipFree(w->d_rep) == hipSuccess) && ok;
    if (w->d_tab_prefill) ok = (hipFree(w->d_tab_prefill) == hipSuccess) && ok;
    if (w->d_tab_tpot) ok = (hipFree(w->d_tab_tpot) == hipSuccess) && ok;
    if (w->d_req) ok = (hipFree(w->d_req) == hipSuccess) && ok;
    if (w->d_scratch) ok = (hipFree(w->d_scratch) == hipSuccess) && ok;
    if (w->d_span) ok = (hipFree(w->d_span) == hipSuccess) && ok;
    if (w->d_span_t) ok = (hipFree(w->d_span_t) == hipSuccess) && ok;
    if (w->d_pair) ok = (hipFree(w->d_pair) == hipSuccess) && ok;
    if (w->d_nominal) ok = (hipFree(w->d_nominal) == hipSuccess) && ok;
    if (w->d_nominal_sums) ok = (hipFree(w->d_nominal_sums) == hipSuccess) && ok;
    if (w->d_pending) ok = (hipFree(w->d_pending) == hipSuccess) && ok;
    if (w->h_stage) ok = (hipHostFree(w->h_stage) == hipSuccess) && ok;
    if (w->d_parent) ok = (hipFree(w->d_parent) == hipSuccess) && ok;
    if (w->d_peak) ok = (hipFree(w->d_peak) == hipSuccess) && ok;
    if (w->d_room) ok = (hipFree(w->d_room) == hipSuccess) && ok;
    if (w->d_rows) ok = (hipFree(w->d_rows) == hipSuccess) && ok;
    if (w->d_req8) ok = (hipFree(w->d_req8) == hipSuccess) && ok;
    if (w->d_split_tab) ok = (hipFree(w->d_split_tab) == hipSuccess) && ok;
    if (w->d_split_queue) ok = (hipFree(w->d_split_queue) == hipSuccess) && ok;
    if (w->d_split_order) ok = (hipFree(w->d_split_order) == hipSuccess) && ok;
    if (w->d_split_scratch) ok = (hipFree(w->d_split_scratch) == hipSuccess) && ok;
    if (w->d_bounds) ok = (hipFree(w->d_bounds) == hipSuccess) && ok;
    if (w->d_tab_pair) ok = (hipFree(w->d_tab_pair) == hipSuccess) && ok;
    delete w->roof;
    delete w;
    return ok ? AP_OK : AP_ERR_DEVICE;
}

}  // extern "C"
