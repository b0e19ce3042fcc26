// Screening: the contention-free tables and record (k_nominal_metrics) and the two slot-ring kernels.
#ifndef AP_SCREEN_HPP
#define AP_SCREEN_HPP

#include "ap_common.hpp"

namespace {

// A record no evaluation can produce (slo_ok <= R - n_rejected always): "not scored yet".
__device__ __forceinline__ bool is_pending(const ap_metrics& m) {
    return m.slo_ok == 0xFFFFFFFFu && m.n_rejected == 0xFFFFFFFFu;
}

// Two words in device memory say whether a call has left any pending mark.  A call uses one of
// them (`mine`): every kernel that writes a pending mark also sets it, and the kernels that only
// look for marks leave at once while it is zero.  The calls of a workload take the words in turn,
// and a call's first kernels clear the word of the call after it (`next`), which nothing else
// touches meanwhile.  A word that was never cleared (a captured call replayed on its own) only
// costs the look at the records.
struct PendingWord {
    uint32_t* mine;
    uint32_t* next;
};
__device__ __forceinline__ void pending_raise(const PendingWord& f) {
    __hip_atomic_store(f.mine, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ bool pending_none(const PendingWord& f) {
    return __hip_atomic_load(f.mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u;
}
__device__ __forceinline__ void pending_clear_next(const PendingWord& f) {
    if (blockIdx.x == 0u && threadIdx.x == 0u) __hip_atomic_store(f.next, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Screening kernel geometry (the tables written below use its lane-major layout).
constexpr uint32_t kScreenWaves = 4;
constexpr uint32_t kScreenThreads = kScreenWaves * kWave;
constexpr uint32_t kScreenBlock = kWave * 8u;     // requests per wavefront per block
constexpr uint32_t kScreenMaxSlots = 64;          // slots per replica worth having
constexpr uint32_t kScreenMinSlots = 32;          // fewer (with B allowing more) and the one-wavefront kernel is not used
constexpr uint32_t kScreenLdsPerWave = 9216;      // bytes of slot state one wavefront may hold

// Position of request r in the lane-major tables: in its block of 512, request
// 128k + 2l + h is element 2k + h of lane l.
__host__ __device__ inline uint32_t screen_table_index(uint32_t r) {
    const uint32_t x = r % kScreenBlock, k = x / 128u, l = (x % 128u) / 2u, h = x % 2u;
    return (r - x) + l * 8u + 2u * k + h;
}

// ----------------------------------------------------------------------------------
// cost tables -> metrics of the contention-free replay (one-time, at ap_costmodel_set)
// ----------------------------------------------------------------------------------
// When every replica has the same coefficients and is available for the whole trace, a
// request that never waits has ttft = prefill, e2e = prefill + decode and the same tpot
// whichever replica it is on.  This kernel evaluates the cost model for every request
// (prefill, tpot, decode of the serve-latency equation's integer stand-in), stores the
// contention-free finish times the screening kernels read (in request order and in the
// lane-major layout), and reduces the values to the record every contention-free candidate
// shares.
// Several workgroups share the trace, two consecutive requests per thread and turn (a pair's table
// word needs both).  Each adds its histograms and sums to a copy in device memory that the host has
// cleared (`g_hist`: three histograms of 32-bit counts; `g_acc`: three 64-bit sums, then the latest
// finish time, the number of requests within the objectives and a count of the workgroups that are
// done); the workgroup that finds itself last takes the totals through the usual reduction.
template <bool kHist16>
__global__ __launch_bounds__(kThreads) void k_nominal_metrics(EvalParams p, uint32_t* __restrict__ span,
                                                              uint32_t* __restrict__ span_t, uint32_t* __restrict__ pair,
                                                              uint32_t tick_us, uint32_t* g_hist, unsigned long long* g_acc,
                                                              ap_metrics* __restrict__ nominal) {
    extern __shared__ __align__(16) unsigned char lds[];
    __shared__ uint32_t finished_before;
    uint32_t* hist = reinterpret_cast<uint32_t*>(lds);
    unsigned long long* acc64 = reinterpret_cast<unsigned long long*>(lds + p.off_misc);
    uint32_t* acc32 = reinterpret_cast<uint32_t*>(lds + p.off_misc + 24);
    uint32_t* wtot = reinterpret_cast<uint32_t*>(lds + p.off_misc + 64);
    uint32_t* g_acc32 = reinterpret_cast<uint32_t*>(g_acc + 3);              // latest finish, within objectives, workgroups done
    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    hist_clear<kHist16>(hist);
    if (tid < 16u) reinterpret_cast<uint32_t*>(acc64)[tid] = 0u;
    __syncthreads();
    const DevReplica rp = p.rep[0];
    unsigned long long s_e2e = 0, s_ttft = 0, s_tpot = 0;
    uint32_t last_fin = 0, n_ok = 0;
    const uint32_t n_pairs = (p.R + 1u) / 2u;
    for (uint32_t q = blockIdx.x * kThreads + tid; q < n_pairs; q += gridDim.x * kThreads) {
        uint32_t word[2] = {0u, 0u};
#pragma unroll
        for (uint32_t h = 0; h < 2u; ++h) {
            const uint32_t r = 2u * q + h;
            if (r < p.R) {
                uint32_t prefill, tpot;
                request_cost(p.tab_prefill, p.tab_tpot, rp, r, p.prompt[r], prefill, tpot);
                const uint32_t e2e = prefill + p.outlen[r] * tpot;
                // service interval in ticks, rounded outwards (arrival down, finish up), 16 bits each
                const uint32_t arrival = p.arrival[r], fin_us = arrival + e2e;
                word[h] = (arrival / tick_us) | ((fin_us ? (fin_us - 1u) / tick_us + 1u : 0u) << 16);
                span[r] = word[h];
                span_t[screen_table_index(r)] = word[h];
                hist_add<kHist16>(hist, 0u, hist_bin_u32(prefill), 1u);
                hist_add<kHist16>(hist, 1u, hist_bin_u32(tpot), 1u);
                hist_add<kHist16>(hist, 2u, hist_bin_u32(e2e), 1u);
                s_ttft += prefill;
                s_e2e += e2e;
                s_tpot += tpot;
                last_fin = max(last_fin, fin_us);
                n_ok += (prefill <= p.slo_ttft && tpot <= p.slo_tpot) ? 1u : 0u;
            }
        }
        // One word per pair of consecutive requests: arrival tick of the first | (finish tick of the
        // first - that arrival) << 16 | (finish tick of the second - that arrival) << 24.  The host
        // asks for this table only with a tick for which both differences are below 256.
        if (pair != nullptr) {
            const uint32_t s0 = word[0], s1 = 2u * q + 1u < p.R ? word[1] : s0;
            const uint32_t arr = s0 & 0xFFFFu;
            pair[q] = arr | (((s0 >> 16) - arr) << 16) | (((s1 >> 16) - arr) << 24);
        }
    }
    // this workgroup's share into the copy in device memory
    s_e2e = wave_sum_u64(s_e2e);
    s_ttft = wave_sum_u64(s_ttft);
    s_tpot = wave_sum_u64(s_tpot);
    last_fin = wave_max_u32(last_fin);
    n_ok = wave_sum_u32(n_ok);
    if (lane == 0u) {
        atomicAdd(&g_acc[0], s_e2e);
        atomicAdd(&g_acc[1], s_ttft);
        atomicAdd(&g_acc[2], s_tpot);
        atomicMax(&g_acc32[0], last_fin);
        atomicAdd(&g_acc32[1], n_ok);
    }
    __syncthreads();                                  // the histograms in LDS are complete
    for (uint32_t i = tid; i < 3u * kBins; i += kThreads) {
        const uint32_t count = hist_get<kHist16>(hist, i / kBins, i % kBins);
        if (count != 0u) atomicAdd(&g_hist[i], count);
    }
    __threadfence();
    __syncthreads();
    if (tid == 0u) finished_before = atomicAdd(&g_acc32[2], 1u);
    __syncthreads();
    if (finished_before != gridDim.x - 1u) return;    // the same word for every thread
    // the last one: every other workgroup's additions were made before it counted itself done
    __threadfence();
    hist_clear<kHist16>(hist);
    if (tid < 16u) reinterpret_cast<uint32_t*>(acc64)[tid] = 0u;
    __syncthreads();
    for (uint32_t i = tid; i < 3u * kBins; i += kThreads) {
        const uint32_t count = __hip_atomic_load(&g_hist[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (count != 0u) hist_add<kHist16>(hist, i / kBins, i % kBins, count);
    }
    unsigned long long t_e2e = 0, t_ttft = 0, t_tpot = 0;
    uint32_t t_last = 0, t_ok = 0;
    if (tid == 0u) {
        t_e2e = __hip_atomic_load(&g_acc[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        t_ttft = __hip_atomic_load(&g_acc[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        t_tpot = __hip_atomic_load(&g_acc[2], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        t_last = __hip_atomic_load(&g_acc32[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        t_ok = __hip_atomic_load(&g_acc32[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    finish_candidate<kHist16>(p, hist, acc64, acc32, wtot, t_e2e, t_ttft, t_tpot, t_last, t_ok, 0u, nominal);
}

// ----------------------------------------------------------------------------------
// screening: prove that a candidate is contention-free without queueing its requests
// ----------------------------------------------------------------------------------
// Applies when every replica has the same coefficients and is available throughout, so a
// request that does not wait occupies a slot during [arrival, arrival + service).
// Each replica gets S <= B screening slots in LDS, all 0.  Every request probes slots of its
// replica with an atomic max of its service interval: a probe whose old value ends at or
// before the request's arrival has claimed a slot that no request still in service at that
// instant holds; any other probe only raises the slot's value.  Slot values never decrease, so
// a slot can look busy when it is not but never free when it is busy: two requests that
// claimed the same slot have disjoint service intervals, in whatever order they were
// processed and whichever slots they tried.  Hence, if every request of the candidate claims a
// slot, the contention-free schedule keeps at most S <= B requests in service per replica at
// any time, nobody waits in the B-slot queue, and the candidate's record is the nominal one.
// The test is sufficient, not necessary: a candidate with a request that finds no slot, or that
// names a replica outside the table, is marked pending and is replayed exactly by
// k_eval_candidates.  Requests are taken roughly in arrival order, which keeps the number of
// slots a replica needs close to its true concurrency.
//
// Times here are 16-bit ticks of 2^k microseconds (k chosen so that the whole range fits),
// with every service interval rounded outwards: arrival down, finish up.  A claim needs
// old finish tick <= arrival tick, which implies old finish <= arrival in microseconds, so
// the rounding only makes the test more conservative; it halves the table bytes read per
// request (one 32-bit span word: arrival tick | finish tick << 16).  In the one-wavefront
// kernel a slot holds the whole span word of its last claimant (the maximum is still ordered
// by finish tick, and the test compares two 16-bit halves, so no field has to be extracted);
// in the eight-wavefront kernel it holds the bare finish tick.
//
// One more ring follows the M real ones in a candidate's slot state: ring M takes the requests
// that name an unknown replica and is kept at "never free", so such a request loses every
// probe and the candidate ends up pending.  The ragged tail passes its absent requests as
// (replica 0, arrival tick 0xFFFF, finish tick 0): a probe that cannot lose and leaves every
// finish tick as it was.
struct ScreenParams {
    const uint32_t* span;         // [R] in request order: arrival tick | finish tick << 16 (interval rounded outwards)
    const uint32_t* span_t;       // [ceil(R/512)*512] the same words in the order given by screen_table_index
    const uint32_t* pair;         // [ceil(R/2)] one word per two requests: arrival tick | two 8-bit tick counts
    const ap_metrics* nominal;
    uint32_t R, M;
    uint32_t slots_log2;          // S = 1 << slots_log2
    uint32_t wave_bytes;          // small tables: LDS bytes of one wavefront's slot state (a multiple of 4 S)
};

struct ScreenRegs {
    uint32_t pair[4];             // two replica ids per word, as stored in the candidate's row
    uint32_t span[8];             // arrival tick | finish tick << 16
};

template <bool kAligned>
__device__ __forceinline__ void screen_fetch(ScreenRegs& g, const ScreenParams& p, const uint16_t* __restrict__ row,
                                             uint32_t i0, uint32_t lane) {
    // Addresses are a uniform base plus a 32-bit byte offset per lane (the host keeps R below 2^30), which
    // costs one 32-bit add per block instead of 64-bit pointer arithmetic per load.
    const char* row_bytes = reinterpret_cast<const char*>(row) + (i0 + 2u * lane) * 2u;
#pragma unroll
    for (uint32_t k = 0; k < 4u; ++k) {
        const uint16_t* at = reinterpret_cast<const uint16_t*>(row_bytes + 256u * k);
        // assignments are read once: stream them past the caches that hold the tables
        if (kAligned) {
            g.pair[k] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(at));
        } else {
            g.pair[k] = (uint32_t)__builtin_nontemporal_load(at) | ((uint32_t)__builtin_nontemporal_load(at + 1) << 16);
        }
    }
    const char* span_bytes = reinterpret_cast<const char*>(p.span_t) + (i0 + lane * 8u) * 4u;
    const uint4 s0 = *reinterpret_cast<const uint4*>(span_bytes);
    const uint4 s1 = *reinterpret_cast<const uint4*>(span_bytes + 16u);
    g.span[0] = s0.x; g.span[1] = s0.y; g.span[2] = s0.z; g.span[3] = s0.w;
    g.span[4] = s1.x; g.span[5] = s1.y; g.span[6] = s1.z; g.span[7] = s1.w;
}

// LDS words addressed by their 32-bit byte address (ring addresses are computed as integers;
// going through the address keeps the ring base out of every access).
typedef __attribute__((address_space(3))) uint32_t lds_word;
__device__ __forceinline__ uint32_t lds_address(const void* p) {
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}
__device__ __forceinline__ uint32_t lds_max_rtn(uint32_t byte_address, uint32_t v) {
    return __hip_atomic_fetch_max((lds_word*)(uintptr_t)byte_address, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
__device__ __forceinline__ uint32_t lds_add_rtn(uint32_t byte_address, uint32_t v) {
    return __hip_atomic_fetch_add((lds_word*)(uintptr_t)byte_address, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// does the interval whose span word is `old` end after the one of `span` begins?
__device__ __forceinline__ bool span_busy(uint32_t old, uint32_t span) { return (old >> 16) > (span & 0xFFFFu); }

// The slow part shared by both kernels: bit k of `open` says that request k of this lane
// (first tried at LDS address `at[k]`, span word `span[k]`) still has no slot, having tried
// the first `tried` alternatives of its ring.  Round by round, every such lane tries the next
// slot of one open request, until each request has a slot or has tried the whole ring.
// Alternatives are reached by flipping address bits in bit-reversed order (half a ring away, a
// quarter, three quarters, ...), which needs the rings aligned to their size.
// Returns true if some request of this lane found no slot.
// kPlain: the slots hold bare finish ticks instead of span words.
template <uint32_t K, bool kPlain>
__device__ __forceinline__ bool screen_search(const uint32_t (&span)[K], const uint32_t (&at)[K], uint32_t open,
                                              uint32_t tried, uint32_t S, uint32_t slots_log2) {
    bool lane_bad = false;
    uint32_t t = tried + 1u;                                                 // next alternative of the request in hand
    while (__ballot(open != 0u) != 0ull) {
        if (open != 0u) {
            const uint32_t k = 31u - (uint32_t)__clz(open);
            uint32_t cur_at = at[0], cur_span = span[0];
#pragma unroll
            for (uint32_t j = 1; j < K; ++j) {
                cur_at = k == j ? at[j] : cur_at;
                cur_span = k == j ? span[j] : cur_span;
            }
            bool placed = false;
            if (t < S) {
                const uint32_t hop = ((__builtin_bitreverse32(t) >> 1) >> (31u - slots_log2)) << 2;
                const uint32_t was = lds_max_rtn(cur_at ^ hop, kPlain ? cur_span >> 16 : cur_span);
                placed = kPlain ? was <= (cur_span & 0xFFFFu) : !span_busy(was, cur_span);
            }
            const bool last = t + 1u >= S;                                   // no other slot of the ring is left
            lane_bad = lane_bad || (!placed && last);
            if (placed || last) { open &= ~(1u << k); t = tried + 1u; } else { ++t; }
        }
    }
    return lane_bad;
}

// Small replica tables: one wavefront per candidate, nothing shared, no barriers.  A block is
// 512 consecutive requests; lane l holds the eight requests i0 + 128k + 2l + h (k = 0..3,
// h = 0..1): four 4-byte loads of assignment pairs, and two 16-byte loads from the table
// stored lane-major.  Step e = 2k + h therefore covers every other request of a 128-request
// window, close enough to arrival order.
// The slot a request tries first is the next one of its replica's ring in turn: a counter per
// replica (LDS, after the rings) is bumped with a returning atomic add, so the requests of
// one replica within a step get different slots and a slot comes up again only after S more
// requests of that replica.  The eight counter bumps of a block are issued back to back, then
// the eight claims (LDS executes them in order, so the steps still see each other's claims).
template <uint32_t K>
__device__ __forceinline__ bool cursor_claim(const uint32_t (&id)[K], const uint32_t (&span)[K], uint32_t ring0_addr,
                                             uint32_t cursor0_addr, uint32_t ring_shift, uint32_t M, uint32_t S,
                                             uint32_t slots_log2) {
    uint32_t key[K], turn[K], at[K], old[K];
#pragma unroll
    for (uint32_t e = 0; e < K; ++e) {
        key[e] = min(id[e], M);                                              // unknown replicas: the never-free ring
        turn[e] = lds_add_rtn(cursor0_addr + (key[e] << 2), 1u);
    }
#pragma unroll
    for (uint32_t e = 0; e < K; ++e) {
        // the replica id is added to the turn: cursors of different replicas advance at much the same pace, and
        // rings are a multiple of the bank count apart, so equal turns would send a whole step to one LDS bank
        at[e] = ring0_addr + (key[e] << ring_shift) + (((turn[e] + key[e]) & (S - 1u)) << 2);
        old[e] = lds_max_rtn(at[e], span[e]);
    }
    bool any = false;
#pragma unroll
    for (uint32_t e = 0; e < K; ++e) any = any || span_busy(old[e], span[e]);
    if (__ballot(any) == 0ull) return false;
    uint32_t open = 0;                                                       // rare: somebody's slot was still taken
#pragma unroll
    for (uint32_t e = 0; e < K; ++e) open |= span_busy(old[e], span[e]) ? 1u << e : 0u;
    return screen_search<K, false>(span, at, open, 0u, S, slots_log2);
}

// kMarked: look only at the candidates whose record already carries the pending mark (the rows
// written for the children that k_certify_children could not settle); every other record is final.
template <bool kAligned, bool kMarked>
__global__ __launch_bounds__(kScreenThreads) void k_screen_candidates(ScreenParams p, const uint16_t* __restrict__ assign,
                                                                       ap_metrics* __restrict__ out, uint32_t C,
                                                                       PendingWord flags) {
    extern __shared__ __align__(16) unsigned char lds[];
    pending_clear_next(flags);
    if (kMarked && pending_none(flags)) return;                              // nobody has left a mark
    const uint32_t lane = threadIdx.x & 63u, w = wave_index();
    const uint32_t M = p.M, R = p.R, S = 1u << p.slots_log2;
    const uint32_t ring_shift = p.slots_log2 + 2u;                           // bytes per ring, log2
    uint32_t* mine = reinterpret_cast<uint32_t*>(lds + w * p.wave_bytes);    // M + 1 rings, then M + 1 counters
    const uint32_t n_ring_words = (M + 1u) << p.slots_log2;
    const uint32_t ring0_addr = lds_address(mine);
    const uint32_t cursor0_addr = ring0_addr + n_ring_words * 4u;
    const uint32_t n_full = R / kScreenBlock;
    const bool rings_aligned = (ring0_addr & ((S << 2) - 1u)) == 0u;

    // kMarked: a workgroup owns a run of consecutive candidates (at most one per thread), looks at all
    // their records at once and leaves when none is marked - the usual case
    uint32_t c_first = blockIdx.x * kScreenWaves, c_end = C, c_step = gridDim.x * kScreenWaves;
    if (kMarked) {
        const uint32_t per = (C + gridDim.x - 1u) / gridDim.x;
        c_first = blockIdx.x * per;
        c_end = min(C, c_first + per);
        c_step = kScreenWaves;
        const uint32_t mine = c_first + threadIdx.x;
        if (__syncthreads_or(threadIdx.x < per && mine < c_end && is_pending(out[mine]) ? 1 : 0) == 0) return;
    }
    for (uint32_t c = c_first + w; c < c_end; c += c_step) {
        if (kMarked && !is_pending(out[c])) continue;
        const uint16_t* row = assign + (size_t)c * R;
        for (uint32_t i = lane; i < n_ring_words + M + 1u; i += kWave)
            mine[i] = (i < n_ring_words && (i >> p.slots_log2) == M) ? kNever : 0u;
        bool bad = !rings_aligned;

        // full blocks, two register sets: one is processed while the other is being loaded
        ScreenRegs ga, gb;
        if (n_full > 0u && !bad) screen_fetch<kAligned>(ga, p, row, 0u, lane);
        for (uint32_t b = 0; b < n_full && !bad; b += 2u) {
            if (b + 1u < n_full) screen_fetch<kAligned>(gb, p, row, (b + 1u) * kScreenBlock, lane);
            {
                const uint32_t id[8] = {ga.pair[0] & 0xFFFFu, ga.pair[0] >> 16, ga.pair[1] & 0xFFFFu, ga.pair[1] >> 16,
                                        ga.pair[2] & 0xFFFFu, ga.pair[2] >> 16, ga.pair[3] & 0xFFFFu, ga.pair[3] >> 16};
                bad = __ballot(cursor_claim<8>(id, ga.span, ring0_addr, cursor0_addr, ring_shift, M, S, p.slots_log2)) != 0ull;
            }
            if (bad || b + 1u >= n_full) break;
            if (b + 2u < n_full) screen_fetch<kAligned>(ga, p, row, (b + 2u) * kScreenBlock, lane);
            {
                const uint32_t id[8] = {gb.pair[0] & 0xFFFFu, gb.pair[0] >> 16, gb.pair[1] & 0xFFFFu, gb.pair[1] >> 16,
                                        gb.pair[2] & 0xFFFFu, gb.pair[2] >> 16, gb.pair[3] & 0xFFFFu, gb.pair[3] >> 16};
                bad = __ballot(cursor_claim<8>(id, gb.span, ring0_addr, cursor0_addr, ring_shift, M, S, p.slots_log2)) != 0ull;
            }
        }

        // ragged tail: the same steps with every access guarded
        const uint32_t i0 = n_full * kScreenBlock;
        if (!bad && i0 < R) {
            uint32_t id[8], span[8];
#pragma unroll
            for (uint32_t e = 0; e < 8u; ++e) {
                const uint32_t r = i0 + 128u * (e >> 1) + 2u * lane + (e & 1u);
                const bool in = r < R;
                id[e] = in ? (uint32_t)row[r] : 0u;
                span[e] = in ? p.span_t[i0 + lane * 8u + e] : 0xFFFFu;       // absent: arrives last, finishes at 0
            }
            bad = __ballot(cursor_claim<8>(id, span, ring0_addr, cursor0_addr, ring_shift, M, S, p.slots_log2)) != 0ull;
        }

        // 64-byte record: nominal, or the pending mark
        if (lane < 8u) {
            const unsigned long long* src = reinterpret_cast<const unsigned long long*>(p.nominal);
            const unsigned long long v = bad ? ~0ull : src[lane];
            reinterpret_cast<unsigned long long*>(&out[c])[lane] = v;
        }
        if (bad && lane == 0u) pending_raise(flags);
    }
}

// Large replica tables: the eight wavefronts of a workgroup share one candidate, which divides
// the LDS held per wavefront by eight, so that enough wavefronts are resident to hide the LDS
// and memory latency.  A block is 1024 consecutive requests; wavefront j takes the two steps
// 128j + 2l + h of it (one 4-byte load of an assignment pair and one 8-byte table load per
// lane), all eight claim from one set of rings, and a barrier per block keeps them within the
// same 1024 requests.  Here lane l tries slot l mod S/2 of the ring first (no counters: with
// eight wavefronts taking turns at random a counter would not keep neighbours apart).
//
// Eight wavefronts work on a block in no particular order, and a request that probes a slot
// after a later request has claimed it loses although it need not (a few percent do).  A
// request that lost goes straight to a slot in the other half of the ring, in the same
// instruction in which the lanes that won send a zero there (which changes nothing), so the
// common case has no branch.  What is left - requests that lost twice - goes through
// screen_search.
constexpr uint32_t kWideWaves = 8;
constexpr uint32_t kWideThreads = kWideWaves * kWave;
constexpr uint32_t kWideBlock = kWideWaves * 128u;
constexpr uint32_t kWideMaxSlots = 64;
constexpr uint32_t kWideLdsBytes = 32768;         // rings of the M real replicas of the one candidate a workgroup holds

// Slots of this kernel hold bare finish ticks.  Is the slot whose old content is `old` still
// taken when the request whose arrival tick is the lower half of `arrival` comes in?
__device__ __forceinline__ bool wide_busy(uint32_t old, uint32_t arrival) { return old > (arrival & 0xFFFFu); }

// Resolve the K first probes of a lane: `old[k]` came back from slot `at[k]`, where the request
// offered its finish tick `finish[k]`; `arrival[k]` is any word whose lower half is the
// request's arrival tick.  Second probe `second[k]` bytes further on for those that lost, then
// the search.  Returns true if some request found no slot in its whole ring.
template <uint32_t K>
__device__ __forceinline__ bool wide_resolve(const uint32_t (&finish)[K], const uint32_t (&arrival)[K],
                                             const uint32_t (&at)[K], const uint32_t (&old)[K],
                                             const uint32_t (&second)[K], uint32_t S, uint32_t slots_log2) {
    uint32_t old2[K];
#pragma unroll
    for (uint32_t k = 0; k < K; ++k) {
        const bool lost = wide_busy(old[k], arrival[k]);
        old2[k] = lds_max_rtn(at[k] + second[k], lost ? finish[k] : 0u);     // a zero changes nothing
    }
    bool any = false;
#pragma unroll
    for (uint32_t k = 0; k < K; ++k) any = any || (wide_busy(old[k], arrival[k]) && wide_busy(old2[k], arrival[k]));
    if (__ballot(any) == 0ull) return false;
    uint32_t open = 0;                                                       // rare: somebody lost twice
    uint32_t span[K];
#pragma unroll
    for (uint32_t k = 0; k < K; ++k) {
        open |= (wide_busy(old[k], arrival[k]) && wide_busy(old2[k], arrival[k])) ? 1u << k : 0u;
        span[k] = (finish[k] << 16) | (arrival[k] & 0xFFFFu);
    }
    return screen_search<K, true>(span, at, open, 0u, S, slots_log2);        // all other slots of the ring, in its usual order
}

// kPacked: the table is read one word per pair of requests (half the bytes of two span words).  The
// second request of a pair is then treated as arriving with the first, which only widens its
// interval.  The host allows it when the tick that makes the 8-bit counts fit is not much
// coarser than the tick the 16-bit fields need.
__device__ __forceinline__ void unpack_pair(uint32_t word, uint32_t& finish0, uint32_t& finish1) {
    finish0 = (word & 0xFFFFu) + ((word >> 16) & 0xFFu);
    finish1 = (word & 0xFFFFu) + (word >> 24);
}

template <bool kAligned, bool kPacked, bool kMarked>
__global__ __launch_bounds__(kWideThreads) void k_screen_candidates_wide(ScreenParams p,
                                                                          const uint16_t* __restrict__ assign,
                                                                          ap_metrics* __restrict__ out, uint32_t C,
                                                                          PendingWord flags) {
    extern __shared__ __align__(16) unsigned char lds[];
    const uint32_t tid = threadIdx.x, lane = tid & 63u, j = wave_index();
    pending_clear_next(flags);
    if (kMarked && pending_none(flags)) return;                              // nobody has left a mark
    const uint32_t M = p.M, R = p.R, S = 1u << p.slots_log2;
    const uint32_t ring_shift = p.slots_log2 + 2u;
    const uint32_t n_words = (M + 1u) << p.slots_log2;                       // M rings and the unknown-replica ring
    uint32_t* slot = reinterpret_cast<uint32_t*>(lds);
    uint32_t* flag = slot + n_words;
    const uint32_t ring0_addr = lds_address(slot);
    // First choices come from the lower half of a ring only, which leaves the upper half (where the
    // second probe goes) to the few requests that lost.  The requests of a block that share a first
    // choice (same lane modulo S/2: two lanes, eight wavefronts, two steps) are sent to different
    // slots of the upper half, so that those of them that go to one replica - the likely losers - do
    // not meet again.
    const uint32_t lower = (S > 1u ? S >> 1 : 1u) - 1u;                      // mask of a slot index in the lower half
    const uint32_t slot_addr = ring0_addr + (lane & lower) * 4u;
    uint32_t second[2];                                                      // from a request's first slot to its second, bytes
#pragma unroll
    for (uint32_t h = 0; h < 2u; ++h)
        second[h] = ((S >> 1) + ((lane + (lane >> 5) + 2u * j + 16u * h) & lower) - (lane & lower)) * 4u;
    const uint32_t n_full = R / kWideBlock;
    const uint32_t mine = 128u * j + 2u * lane;                              // offset of this lane's pair in a block
    // alternatives are reached by flipping address bits, which needs the rings aligned to their size
    const bool rings_aligned = (ring0_addr & ((S << 2) - 1u)) == 0u;

    // kMarked: a workgroup owns a run of consecutive candidates (at most one per thread), looks at all
    // their records at once and leaves when none is marked - the usual case
    uint32_t c_first = blockIdx.x, c_end = C, c_step = gridDim.x;
    if (kMarked) {
        const uint32_t per = (C + gridDim.x - 1u) / gridDim.x;
        c_first = blockIdx.x * per;
        c_end = min(C, c_first + per);
        c_step = 1u;
        if (__syncthreads_or(tid < per && c_first + tid < c_end && is_pending(out[c_first + tid]) ? 1 : 0) == 0) return;
    }
    for (uint32_t c = c_first; c < c_end; c += c_step) {
        if (kMarked && !is_pending(out[c])) continue;                        // the same for the whole workgroup
        const uint16_t* row = assign + (size_t)c * R;
        for (uint32_t i = tid; i < n_words; i += kWideThreads) slot[i] = (i >> p.slots_log2) == M ? kNever : 0u;
        if (tid < 2u) flag[tid] = rings_aligned ? 0u : 1u;
        __syncthreads();

        // Full blocks go in groups of kDepth.  While a group is processed the loads of the next
        // group are issued, one register per block and stream, so kDepth blocks stay in flight per
        // wavefront; the body is straight-line (the prefetch index is clamped instead of
        // guarded), and two register sets take turns (a group loads into the set it does not
        // read), so nothing has to be copied, or waited for, between groups.  The verdict is
        // exchanged once per group: group g reports in flag[g & 1], and a wavefront already in
        // the next group writes the other word, so all wavefronts read the same verdict and
        // leave together.
        constexpr uint32_t kDepth = 4;
        struct Loaded {
            uint32_t pair[kDepth];    // two replica ids
            uint2 span[kDepth];       // their table words (.x only when packed)
        };
        auto fetch = [&](Loaded& into, uint32_t d, uint32_t blk) {
            // A uniform base plus a 32-bit byte offset per lane (the host keeps R below 2^30): the pair of
            // ids and the pair's table word sit at the same offset, so one 32-bit add serves both loads.
            const uint32_t off = (blk * kWideBlock + mine) * 2u;
            const uint16_t* at = reinterpret_cast<const uint16_t*>(reinterpret_cast<const char*>(row) + off);
            if (kAligned) {
                into.pair[d] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(at));
            } else {
                into.pair[d] = (uint32_t)__builtin_nontemporal_load(at) | ((uint32_t)__builtin_nontemporal_load(at + 1) << 16);
            }
            if (kPacked) {
                into.span[d].x = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const char*>(p.pair) + off);
            } else {
                into.span[d] = *reinterpret_cast<const uint2*>(reinterpret_cast<const char*>(p.span) + off * 2u);
            }
        };
        auto first_probe = [&](uint32_t id, uint32_t finish, uint32_t& at, uint32_t& old) {
            at = (min(id, M) << ring_shift) + slot_addr;                     // unknown replicas: the never-free ring
            old = lds_max_rtn(at, finish);
        };
        const uint32_t n_groups = n_full / kDepth;
        bool bad = !rings_aligned;
        uint32_t turn = 0;                                                   // which flag word the next verdict uses
        auto run_group = [&](const Loaded& now, Loaded& next, uint32_t g) {
            bool lane_bad = false;
#pragma unroll
            for (uint32_t d = 0; d < kDepth; ++d) {
                uint32_t value[2], arrival[2], at[2], old[2];
                const uint32_t ids = now.pair[d];
                if (kPacked) {
                    unpack_pair(now.span[d].x, value[0], value[1]);
                    arrival[0] = arrival[1] = now.span[d].x;                 // the pair's arrival tick is its lower half
                } else {
                    arrival[0] = now.span[d].x;
                    arrival[1] = now.span[d].y;
                    value[0] = arrival[0] >> 16;
                    value[1] = arrival[1] >> 16;
                }
                fetch(next, d, min((g + 1u) * kDepth + d, n_full - 1u));     // redundant in the last group
                first_probe(ids & 0xFFFFu, value[0], at[0], old[0]);
                first_probe(ids >> 16, value[1], at[1], old[1]);
                lane_bad = wide_resolve<2>(value, arrival, at, old, second, S, p.slots_log2) || lane_bad;
                if (d + 1u < kDepth) __syncthreads();
            }
            if (__ballot(lane_bad) != 0ull && lane == 0) flag[turn & 1u] = 1u;
            __syncthreads();
            bad = flag[turn & 1u] != 0u;
            ++turn;
        };
        Loaded set_a, set_b;
        if (n_groups > 0u && !bad) {
#pragma unroll
            for (uint32_t d = 0; d < kDepth; ++d) fetch(set_a, d, d);
        }
        uint32_t g = 0;
        for (; g + 2u <= n_groups && !bad; g += 2u) {
            run_group(set_a, set_b, g);
            if (!bad) run_group(set_b, set_a, g + 1u);
        }
        if (g < n_groups && !bad) run_group(set_a, set_b, g);               // an odd number of groups
        // fewer than kDepth full blocks left, then the ragged tail with every access guarded
        // (an absent request is a probe of replica 0 that changes nothing and cannot lose)
        const uint32_t n_rest = n_full - n_groups * kDepth + (n_full * kWideBlock < R ? 1u : 0u);
        for (uint32_t k = 0; k < n_rest && !bad; ++k, ++turn) {
            const uint32_t i0 = (n_groups * kDepth + k) * kWideBlock;
            uint32_t sp[2], fin[2], at[2], old[2];
#pragma unroll
            for (uint32_t h = 0; h < 2u; ++h) {
                const uint32_t r = i0 + mine + h;
                const bool in = r < R;
                sp[h] = 0xFFFFu;                                             // absent: arrives last, finishes at 0
                fin[h] = 0u;
                if (in && kPacked) {
                    const uint32_t word = p.pair[r >> 1];
                    uint32_t both[2];
                    unpack_pair(word, both[0], both[1]);
                    sp[h] = word;
                    fin[h] = both[h];
                } else if (in) {
                    sp[h] = p.span[r];
                    fin[h] = sp[h] >> 16;
                }
                first_probe(in ? (uint32_t)row[r] : 0u, fin[h], at[h], old[h]);
            }
            const bool lane_bad = wide_resolve<2>(fin, sp, at, old, second, S, p.slots_log2);
            if (__ballot(lane_bad) != 0ull && lane == 0) flag[turn & 1u] = 1u;
            __syncthreads();
            bad = flag[turn & 1u] != 0u;
        }
        if (tid < 8u) {
            const unsigned long long* src = reinterpret_cast<const unsigned long long*>(p.nominal);
            reinterpret_cast<unsigned long long*>(&out[c])[tid] = bad ? ~0ull : src[tid];
        }
        if (bad && tid == 0u) pending_raise(flags);
        __syncthreads();                                                     // everyone has read the flags
    }
}

}  // namespace

#endif  // AP_SCREEN_HPP
