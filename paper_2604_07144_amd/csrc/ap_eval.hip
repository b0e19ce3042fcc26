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
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstring>
#include <new>
#include <type_traits>
#include <vector>

#include "autopoiesis_eval.h"

namespace {

constexpr uint32_t kWave = 64;
constexpr uint32_t kWaves = 8;                  // wavefronts per workgroup
constexpr uint32_t kThreads = kWave * kWaves;   // 512
constexpr uint32_t kBins = 4096;
constexpr uint32_t kBinsPerThread = kBins / kThreads;
constexpr uint32_t kMaxGroups = 8;              // 64-request groups per wavefront per chunk
constexpr uint32_t kMaxChunk = kThreads * kMaxGroups;
constexpr uint32_t kNever = 0xFFFFFFFFu;        // "no such time": larger than every reachable time
constexpr uint32_t kNoKey = 0xFFFFFFFFu;

struct DevReplica {
    uint32_t a, b, c, d;      // cost coefficients
    uint32_t t_on, t_off;     // window, relative microseconds (t_off == kNever: never leaves)
};

struct EvalParams {
    const uint32_t* arrival;  // [R] relative microseconds
    const uint32_t* prompt;   // [R]
    const uint32_t* outlen;   // [R]
    const DevReplica* rep;    // [M]
    uint32_t R, M, B, chunk, key_bits;
    uint32_t slo_ttft, slo_tpot;
    uint32_t penalty_bin, k99;
    uint64_t penalty;
    // byte offsets into dynamic LDS
    uint32_t off_slots, off_sorted, off_close, off_cnt, off_qstart, off_list, off_arr, off_prompt, off_out, off_misc;
};

// ----------------------------------------------------------------------------------
// wavefront helpers (64 lanes)
// ----------------------------------------------------------------------------------
// Index of this wavefront in its workgroup, as a wave-uniform (scalar) value: loops and
// table lookups that depend on it then stay on the scalar unit.
__device__ __forceinline__ uint32_t wave_index() {
    return (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
}

__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v, uint32_t lane) {
#pragma unroll
    for (uint32_t d = 1; d < kWave; d <<= 1) {
        uint32_t t = (uint32_t)__shfl_up((int)v, d);
        if (lane >= d) v += t;
    }
    return v;
}

__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
#pragma unroll
    for (uint32_t d = 32; d >= 1; d >>= 1) v += (uint32_t)__shfl_xor((int)v, d);
    return v;
}

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
#pragma unroll
    for (uint32_t d = 32; d >= 1; d >>= 1) v = max(v, (uint32_t)__shfl_xor((int)v, d));
    return v;
}

__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long v) {
#pragma unroll
    for (uint32_t d = 32; d >= 1; d >>= 1) v += (unsigned long long)__shfl_xor((long long)v, d);
    return v;
}

// 4096-bin log-linear histogram map for values below 2^32.
__device__ __forceinline__ uint32_t hist_bin_u32(uint32_t v) {
    // With s = max(floor(log2 v), 7) - 7 the bin is (s << 7) + (v >> s): below 128 that is v itself, above it
    // v >> s lies in [128, 256), which supplies both the sub-bin and the +1 of the octave number.
    const uint32_t s = 24u - min((uint32_t)__clz((int)v), 24u);             // __clz(0) is 32
    return (s << 7) + (v >> s);
}

__device__ __forceinline__ unsigned long long hist_lower_edge(uint32_t bin) {
    if (bin < 128u) return bin;
    return (unsigned long long)(128u | (bin & 127u)) << ((bin >> 7) - 1u);
}

// Ascending bitonic sort of one value per lane across the wavefront.
__device__ __forceinline__ uint32_t wave_sort_ascending(uint32_t v, uint32_t lane) {
#pragma unroll
    for (uint32_t k = 2; k <= kWave; k <<= 1) {
#pragma unroll
        for (uint32_t j = k >> 1; j > 0; j >>= 1) {
            const uint32_t other = (uint32_t)__shfl_xor((int)v, (int)j);
            const bool keep_min = ((lane & j) == 0u) == ((lane & k) == 0u);
            v = keep_min ? min(v, other) : max(v, other);
        }
    }
    return v;
}

// Lane i receives lane i + 1's value; lane 63 receives `last`.
__device__ __forceinline__ uint32_t wave_shift_down(uint32_t v, uint32_t last) {
    return (uint32_t)__builtin_amdgcn_update_dpp((int)last, (int)v, 0x130 /* wave_shl:1 */, 0xF, 0xF, false);
}

// The lanes of this wavefront whose key equals mine, as the two halves of a 64-bit mask, for
// the lanes whose key is below `n_keys` (the others get a meaningless mask): one ballot per bit
// of n_keys - 1; a lane keeps the lanes that agree with it on that bit.
__device__ __forceinline__ void wave_peers(uint32_t key, uint32_t n_keys, uint32_t key_bits, uint32_t& lo, uint32_t& hi) {
    const unsigned long long ranked = __ballot(key < n_keys);
    lo = (uint32_t)ranked;
    hi = (uint32_t)(ranked >> 32);
    for (uint32_t b = 0; b < key_bits; ++b) {
        const uint32_t mine = (uint32_t)__builtin_amdgcn_sbfe((int)key, b, 1u);  // all ones if my bit b is set, else 0
        const unsigned long long set = __ballot(mine != 0u);
        lo &= ~((uint32_t)set ^ mine);                                         // lanes whose bit equals mine
        hi &= ~((uint32_t)(set >> 32) ^ mine);
    }
}

// lane i takes lane i - 1's value; lane 0 takes `first`
__device__ __forceinline__ uint32_t wave_shift_up(uint32_t v, uint32_t first) {
    return (uint32_t)__builtin_amdgcn_update_dpp((int)first, (int)v, 0x138 /* wave_shr:1 */, 0xF, 0xF, false);
}

// The three 4096-bin histograms of a candidate in LDS.  When R < 65536 no count can exceed 16
// bits, so two bins share a 32-bit word (half the LDS, half the clearing and scanning).
template <bool kHist16>
__device__ __forceinline__ void hist_add(uint32_t* hist, uint32_t which, uint32_t bin, uint32_t count) {
    if (kHist16) atomicAdd(&hist[which * (kBins / 2u) + (bin >> 1)], count << ((bin & 1u) << 4));
    else atomicAdd(&hist[which * kBins + bin], count);
}

template <bool kHist16>
__device__ __forceinline__ uint32_t hist_get(const uint32_t* hist, uint32_t which, uint32_t bin) {
    if (kHist16) return (hist[which * (kBins / 2u) + (bin >> 1)] >> ((bin & 1u) << 4)) & 0xFFFFu;
    return hist[which * kBins + bin];
}

template <bool kHist16>
__device__ __forceinline__ void hist_clear(uint32_t* hist) {
    for (uint32_t i = threadIdx.x; i < (kHist16 ? 3u * kBins / 2u : 3u * kBins); i += kThreads) hist[i] = 0u;
}

// Block-wide end of one candidate: fold the per-lane sums, add the rejected requests at the
// penalty value, find the three p99 bins by a prefix sum over the histograms and write the
// record.  Called by all kThreads threads; `hist` holds the served requests' counts.
template <bool kHist16>
__device__ __forceinline__ void finish_candidate(const EvalParams& p, uint32_t* hist, unsigned long long* acc64,
                                                 uint32_t* acc32, uint32_t* wtot, unsigned long long s_e2e,
                                                 unsigned long long s_ttft, unsigned long long s_tpot,
                                                 uint32_t last_fin, uint32_t n_ok, uint32_t n_rej,
                                                 ap_metrics* __restrict__ dst) {
    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    const uint32_t w = wave_index();
    s_e2e = wave_sum_u64(s_e2e);
    s_ttft = wave_sum_u64(s_ttft);
    s_tpot = wave_sum_u64(s_tpot);
    last_fin = wave_max_u32(last_fin);
    n_ok = wave_sum_u32(n_ok);
    n_rej = wave_sum_u32(n_rej);
    if (lane == 0) {
        atomicAdd(&acc64[0], s_e2e);
        atomicAdd(&acc64[1], s_ttft);
        atomicAdd(&acc64[2], s_tpot);
        atomicMax(&acc32[0], last_fin);
        atomicAdd(&acc32[1], n_ok);
        atomicAdd(&acc32[2], n_rej);
    }
    __syncthreads();
    const uint32_t rejected = acc32[2];
    if (tid < 3u && rejected) hist_add<kHist16>(hist, tid, p.penalty_bin, rejected);
    __syncthreads();

    // p99: block-wide prefix sum over the bins, kBinsPerThread bins per thread, three histograms at once
    uint32_t part[3], incl[3];
#pragma unroll
    for (uint32_t h = 0; h < 3u; ++h) {
        part[h] = 0;
#pragma unroll
        for (uint32_t i = 0; i < kBinsPerThread; ++i) part[h] += hist_get<kHist16>(hist, h, kBinsPerThread * tid + i);
        incl[h] = wave_inclusive_scan(part[h], lane);
        if (lane == 63u) wtot[h * kWaves + w] = incl[h];
    }
    __syncthreads();
#pragma unroll
    for (uint32_t h = 0; h < 3u; ++h) {
        uint32_t before = 0;
        for (uint32_t ww = 0; ww < w; ++ww) before += wtot[h * kWaves + ww];
        const uint32_t hi = before + incl[h], lo = hi - part[h];
        if (lo < p.k99 && p.k99 <= hi) {
            uint32_t run = lo, b = 0;
            for (; b + 1u < kBinsPerThread; ++b) {
                run += hist_get<kHist16>(hist, h, kBinsPerThread * tid + b);
                if (run >= p.k99) break;
            }
            acc32[3 + h] = kBinsPerThread * tid + b;
        }
    }
    __syncthreads();
    if (tid == 0) {
        ap_metrics mt;
        mt.sum_e2e_us = acc64[0] + (unsigned long long)rejected * p.penalty;
        mt.sum_ttft_us = acc64[1] + (unsigned long long)rejected * p.penalty;
        mt.sum_tpot_us = acc64[2] + (unsigned long long)rejected * p.penalty;
        mt.makespan_us = acc32[0];
        mt.p99_ttft_us = hist_lower_edge(acc32[3]);
        mt.p99_tpot_us = hist_lower_edge(acc32[4]);
        mt.p99_e2e_us = hist_lower_edge(acc32[5]);
        mt.slo_ok = acc32[1];
        mt.n_rejected = rejected;
        *dst = mt;
    }
}

// A record no evaluation can produce (slo_ok <= R - n_rejected always): "not scored yet".
__device__ __forceinline__ bool is_pending(const ap_metrics& m) {
    return m.slo_ok == 0xFFFFFFFFu && m.n_rejected == 0xFFFFFFFFu;
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
// One workgroup.
template <bool kHist16>
__global__ __launch_bounds__(kThreads) void k_nominal_metrics(EvalParams p, uint32_t* span, uint32_t* __restrict__ span_t,
                                                              uint32_t* __restrict__ pair, uint32_t tick_us,
                                                              ap_metrics* __restrict__ nominal) {
    extern __shared__ __align__(16) unsigned char lds[];
    uint32_t* hist = reinterpret_cast<uint32_t*>(lds);
    unsigned long long* acc64 = reinterpret_cast<unsigned long long*>(lds + p.off_misc);
    uint32_t* acc32 = reinterpret_cast<uint32_t*>(lds + p.off_misc + 24);
    uint32_t* wtot = reinterpret_cast<uint32_t*>(lds + p.off_misc + 64);
    const uint32_t tid = threadIdx.x;
    hist_clear<kHist16>(hist);
    if (tid < 16u) reinterpret_cast<uint32_t*>(acc64)[tid] = 0u;
    __syncthreads();
    const DevReplica rp = p.rep[0];
    unsigned long long s_e2e = 0, s_ttft = 0, s_tpot = 0;
    uint32_t last_fin = 0, n_ok = 0;
    for (uint32_t r = tid; r < p.R; r += kThreads) {
        const uint32_t prm = p.prompt[r];
        const uint32_t prefill = rp.a + rp.b * prm;
        const uint32_t tpot = rp.c + rp.d * ((prm + 1023u) >> 10);
        const uint32_t e2e = prefill + p.outlen[r] * tpot;
        // service interval in ticks, rounded outwards (arrival down, finish up), 16 bits each
        const uint32_t fin_us = p.arrival[r] + e2e;
        const uint32_t span_v = (p.arrival[r] / tick_us) | ((fin_us ? (fin_us - 1u) / tick_us + 1u : 0u) << 16);
        span[r] = span_v;
        span_t[screen_table_index(r)] = span_v;
        hist_add<kHist16>(hist, 0u, hist_bin_u32(prefill), 1u);
        hist_add<kHist16>(hist, 1u, hist_bin_u32(tpot), 1u);
        hist_add<kHist16>(hist, 2u, hist_bin_u32(e2e), 1u);
        s_ttft += prefill;
        s_e2e += e2e;
        s_tpot += tpot;
        last_fin = max(last_fin, p.arrival[r] + e2e);
        n_ok += (prefill <= p.slo_ttft && tpot <= p.slo_tpot) ? 1u : 0u;
    }
    finish_candidate<kHist16>(p, hist, acc64, acc32, wtot, s_e2e, s_ttft, s_tpot, last_fin, n_ok, 0u, nominal);
    // One word per pair of consecutive requests: arrival tick of the first | (finish tick of the
    // first - that arrival) << 16 | (finish tick of the second - that arrival) << 24.  The host
    // asks for this table only with a tick for which both differences are below 256.
    if (pair != nullptr) {
        __syncthreads();                              // the span words written above, by this workgroup
        for (uint32_t q = tid; 2u * q < p.R; q += kThreads) {
            const uint32_t s0 = span[2u * q];
            const uint32_t s1 = 2u * q + 1u < p.R ? span[2u * q + 1u] : s0;
            const uint32_t arr = s0 & 0xFFFFu;
            pair[q] = arr | (((s0 >> 16) - arr) << 16) | (((s1 >> 16) - arr) << 24);
        }
    }
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
#pragma unroll
    for (uint32_t k = 0; k < 4u; ++k) {
        const uint16_t* at = row + i0 + 128u * k + 2u * lane;
        // assignments are read once: stream them past the caches that hold the tables
        if (kAligned) {
            g.pair[k] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(at));
        } else {
            g.pair[k] = (uint32_t)__builtin_nontemporal_load(at) | ((uint32_t)__builtin_nontemporal_load(at + 1) << 16);
        }
    }
    const uint4 s0 = *reinterpret_cast<const uint4*>(p.span_t + i0 + lane * 8u);
    const uint4 s1 = *reinterpret_cast<const uint4*>(p.span_t + i0 + lane * 8u + 4u);
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
        at[e] = ring0_addr + (key[e] << ring_shift) + ((turn[e] & (S - 1u)) << 2);
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
                                                                       ap_metrics* __restrict__ out, uint32_t C) {
    extern __shared__ __align__(16) unsigned char lds[];
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
                                                                          ap_metrics* __restrict__ out, uint32_t C) {
    extern __shared__ __align__(16) unsigned char lds[];
    const uint32_t tid = threadIdx.x, lane = tid & 63u, j = wave_index();
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
            const uint32_t i0 = blk * kWideBlock;
            const uint16_t* at = row + i0 + mine;
            if (kAligned) {
                into.pair[d] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(at));
            } else {
                into.pair[d] = (uint32_t)__builtin_nontemporal_load(at) | ((uint32_t)__builtin_nontemporal_load(at + 1) << 16);
            }
            if (kPacked) {
                into.span[d].x = (p.pair + (i0 >> 1))[mine >> 1];
            } else {
                into.span[d] = *reinterpret_cast<const uint2*>(p.span + i0 + mine);
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
        __syncthreads();                                                     // everyone has read the flags
    }
}

// ----------------------------------------------------------------------------------
// the evaluation kernel (exact replay)
// ----------------------------------------------------------------------------------
// only_pending != 0: score just the candidates whose record carries the "still to do" mark
// left by the screening kernel; every other record is final and is not touched.
//
// Replay of one replica's queue segment, 64 requests at a time (one per lane), with the B
// slot-free times one per lane:
//  * if at least as many slots are free at the first request's ready time as there are
//    requests, every request starts when it is ready (free slots stay free for later
//    requests because ready times do not decrease) and the finish times are routed to the
//    free lanes in one permute;
//  * otherwise the requests are taken one by one with the slot times kept sorted across the
//    lanes: lane 0 holds the earliest-free slot, start = max(ready, lane 0), and the new
//    finish time is inserted by one shift-and-compare (new[i] = min(S[i+1], max(S[i], f))).
//    The slots are sorted (bitonic, across lanes) when this mode is entered after a
//    permute-mode update.
//
// kLen16: every prompt and output length is below 65536, so the staged copies are 16-bit.
template <bool kHist16, bool kLen16>
__global__ __launch_bounds__(kThreads) void k_eval_candidates(EvalParams p, const uint16_t* __restrict__ assign,
                                                              ap_metrics* out, uint32_t C, uint32_t only_pending) {
    using len_t = typename std::conditional<kLen16, uint16_t, uint32_t>::type;
    extern __shared__ __align__(16) unsigned char lds[];
    uint32_t* hist = reinterpret_cast<uint32_t*>(lds);                        // three histograms
    uint32_t* slots = reinterpret_cast<uint32_t*>(lds + p.off_slots);         // [M][B] slot-free times
    uint32_t* sorted = reinterpret_cast<uint32_t*>(lds + p.off_sorted);       // [M] slots ascending across lanes?
    uint32_t* cnt = reinterpret_cast<uint32_t*>(lds + p.off_cnt);             // [kWaves][M+1]
    uint32_t* qstart = reinterpret_cast<uint32_t*>(lds + p.off_qstart);       // [M+2]
    uint16_t* list = reinterpret_cast<uint16_t*>(lds + p.off_list);           // [chunk] indices by replica
    uint32_t* c_arr = reinterpret_cast<uint32_t*>(lds + p.off_arr);           // [chunk] staged trace
    len_t* c_prompt = reinterpret_cast<len_t*>(lds + p.off_prompt);
    len_t* c_out = reinterpret_cast<len_t*>(lds + p.off_out);
    uint32_t* t_close = reinterpret_cast<uint32_t*>(lds + p.off_close);       // [M+1] t_off per replica, 0 for "no replica"
    unsigned long long* acc64 = reinterpret_cast<unsigned long long*>(lds + p.off_misc);   // e2e, ttft, tpot
    uint32_t* acc32 = reinterpret_cast<uint32_t*>(lds + p.off_misc + 24);     // makespan, slo_ok, n_rej, p99 bins[3]
    uint32_t* wtot = reinterpret_cast<uint32_t*>(lds + p.off_misc + 64);      // [3][kWaves] scan carries
    uint32_t* next_m = reinterpret_cast<uint32_t*>(lds + p.off_misc + 48);    // next replica nobody has replayed yet

    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    const uint32_t w = wave_index();
    const uint32_t R = p.R, M = p.M, B = p.B, M1 = p.M + 1u;
    const uint32_t grab = max(1u, M / (8u * kWaves));  // replicas a wavefront takes at a time
    for (uint32_t m = tid; m <= M; m += kThreads) t_close[m] = m < M ? p.rep[m].t_off : 0u;
    const uint32_t per_wave = p.chunk / kWaves;       // multiple of 64
    const uint32_t groups = per_wave / kWave;         // <= kMaxGroups
    const unsigned long long lanes_below = (1ull << lane) - 1ull;

    // After screening, most workgroups have nothing left to do: look at all of this workgroup's
    // records at once (one per thread) and leave if none carries the mark.
    if (only_pending) {
        bool any = false;
        for (unsigned long long c = (unsigned long long)blockIdx.x + (unsigned long long)tid * gridDim.x; c < C;
             c += (unsigned long long)kThreads * gridDim.x)
            any = any || is_pending(out[c]);
        if (tid == 0) *next_m = 0u;                   // borrowed as the workgroup's "something to do" word
        __syncthreads();
        if (any) *next_m = 1u;
        __syncthreads();
        if (*next_m == 0u) return;                    // the same word for every thread: all leave or none
    }

    for (uint32_t c = blockIdx.x; c < C; c += gridDim.x) {
        if (only_pending && !is_pending(out[c])) continue;      // same record for every thread: uniform
        const uint16_t* row = assign + (size_t)c * R;

        hist_clear<kHist16>(hist);
        for (uint32_t i = tid; i < M * B; i += kThreads) slots[i] = 0u;
        for (uint32_t i = tid; i < M; i += kThreads) sorted[i] = 1u;       // all zero is sorted
        for (uint32_t i = tid; i < kWaves * M1; i += kThreads) cnt[i] = 0u;
        if (tid < 16u) reinterpret_cast<uint32_t*>(acc64)[tid] = 0u;
        unsigned long long s_e2e = 0, s_ttft = 0, s_tpot = 0;
        uint32_t last_fin = 0, n_ok = 0, n_rej = 0;
        __syncthreads();

        // Each thread owns the same positions of every chunk: position w * per_wave + 64 g + lane
        // for g < groups.  Their assignment ids and arrival times are loaded one chunk ahead.
        uint32_t key[kMaxGroups], karr[kMaxGroups];
        auto load_keys = [&](uint32_t r0) {
            const uint32_t n = r0 < R ? min(p.chunk, R - r0) : 0u;
#pragma unroll
            for (uint32_t g = 0; g < kMaxGroups; ++g) {
                const uint32_t idx = w * per_wave + g * kWave + lane;
                const bool in = g < groups && idx < n;
                key[g] = in ? (uint32_t)row[r0 + idx] : kNoKey;
                karr[g] = in ? p.arrival[r0 + idx] : 0u;
            }
        };
        load_keys(0u);

        for (uint32_t r0 = 0; r0 < R; r0 += p.chunk) {
            // ---- stage the chunk of the trace (lengths are written to LDS after the scatter) -
            uint32_t kprompt[kMaxGroups], kout[kMaxGroups];
#pragma unroll
            for (uint32_t g = 0; g < kMaxGroups; ++g) {
                if (key[g] == kNoKey) continue;
                const uint32_t idx = w * per_wave + g * kWave + lane;
                kprompt[g] = p.prompt[r0 + idx];
                kout[g] = p.outlen[r0 + idx];
                c_arr[idx] = karr[g];
                // a request that arrives when its replica is already gone can never start: reject it
                // here (key M, like an unknown replica) instead of queueing it
                const uint32_t k = min(key[g], M);
                key[g] = karr[g] >= t_close[k] ? M : k;
            }

            // ---- (1) per-wavefront replica histogram (cnt was cleared during the last replay) --
#pragma unroll
            for (uint32_t g = 0; g < kMaxGroups; ++g)
                if (key[g] != kNoKey) atomicAdd(&cnt[w * M1 + key[g]], 1u);
            __syncthreads();

            // ---- (2) offsets: down the wavefronts per replica, then across replicas --------
            if (M1 <= 2u * kWave) {                   // few replicas: one wavefront does both
                if (w == 0) {
                    uint32_t carry = 0;
                    for (uint32_t base = 0; base <= M; base += kWave) {
                        const uint32_t m = base + lane;
                        uint32_t run = 0;
                        if (m <= M) {
                            for (uint32_t ww = 0; ww < kWaves; ++ww) {
                                const uint32_t t = cnt[ww * M1 + m];
                                cnt[ww * M1 + m] = run;
                                run += t;
                            }
                        }
                        const uint32_t incl = wave_inclusive_scan(run, lane);
                        if (m <= M) qstart[m] = carry + incl - run;
                        carry += (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
                    }
                    if (lane == 0) qstart[M1] = carry;
                }
            } else {
                for (uint32_t m = tid; m <= M; m += kThreads) {
                    uint32_t run = 0;
                    for (uint32_t ww = 0; ww < kWaves; ++ww) {
                        uint32_t t = cnt[ww * M1 + m];
                        cnt[ww * M1 + m] = run;
                        run += t;
                    }
                    qstart[m] = run;
                }
                __syncthreads();
                if (w == 0) {
                    uint32_t carry = 0;
                    for (uint32_t base = 0; base <= M; base += kWave) {
                        uint32_t m = base + lane;
                        uint32_t v = m <= M ? qstart[m] : 0u;
                        uint32_t incl = wave_inclusive_scan(v, lane);
                        if (m <= M) qstart[m] = carry + incl - v;
                        carry += (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
                    }
                    if (lane == 0) qstart[M1] = carry;
                }
            }
            __syncthreads();

            // ---- (3) stable scatter: rank among equal keys of the group by ballots ---------
#pragma unroll
            for (uint32_t g = 0; g < kMaxGroups; ++g) {
                if (g >= groups) break;
                const uint32_t k = key[g];
                uint32_t peers_lo, peers_hi;
                wave_peers(k, M, p.key_bits, peers_lo, peers_hi);
                if (k < M) {
                    const uint32_t rank = __builtin_amdgcn_mbcnt_hi(peers_hi, __builtin_amdgcn_mbcnt_lo(peers_lo, 0u));
                    const uint32_t total = __popc(peers_lo) + __popc(peers_hi);
                    uint32_t base = qstart[k] + cnt[w * M1 + k];
                    list[base + rank] = (uint16_t)(w * per_wave + g * kWave + lane);
                    if (rank + 1u == total) cnt[w * M1 + k] += total;
                } else if (k == M) {
                    n_rej += 1u;        // no such replica, or it left before the request arrived
                }
                if (k != kNoKey) {
                    const uint32_t idx = w * per_wave + g * kWave + lane;
                    c_prompt[idx] = (len_t)kprompt[g];
                    c_out[idx] = (len_t)kout[g];
                }
            }
            if (tid == 0) *next_m = 0u;
            __syncthreads();
            // the next chunk's assignments and arrival times arrive while this one is replayed
            load_keys(r0 + p.chunk);
            for (uint32_t i = tid; i < kWaves * M1; i += kThreads) cnt[i] = 0u;

            // ---- (4)+(5) replay: one wavefront per replica, lanes = slots / requests ------
            // Queue lengths differ a lot between replicas (a replica that has just come up has
            // its whole backlog to serve one by one), so the wavefronts take replicas from a
            // shared counter instead of a fixed share.
            for (;;) {
                uint32_t m_first = 0;
                if (lane == 0) m_first = atomicAdd(next_m, grab);
                m_first = (uint32_t)__builtin_amdgcn_readfirstlane((int)m_first);
                if (m_first >= M) break;
            for (uint32_t m = m_first; m < min(m_first + grab, M); ++m) {
                const uint32_t qs = qstart[m];
                const uint32_t qn = qstart[m + 1] - qs;
                if (qn == 0) continue;
                // the replica's parameters are the same for every lane: keep them on the scalar unit
                DevReplica rp = p.rep[m];
                rp.a = (uint32_t)__builtin_amdgcn_readfirstlane((int)rp.a);
                rp.b = (uint32_t)__builtin_amdgcn_readfirstlane((int)rp.b);
                rp.c = (uint32_t)__builtin_amdgcn_readfirstlane((int)rp.c);
                rp.d = (uint32_t)__builtin_amdgcn_readfirstlane((int)rp.d);
                rp.t_on = (uint32_t)__builtin_amdgcn_readfirstlane((int)rp.t_on);
                rp.t_off = (uint32_t)__builtin_amdgcn_readfirstlane((int)rp.t_off);
                uint32_t S = lane < B ? slots[m * B + lane] : kNever;
                bool in_order = __builtin_amdgcn_readfirstlane((int)sorted[m]) != 0;
                for (uint32_t sb = 0; sb < qn; sb += kWave) {
                    const uint32_t nb = min(kWave, qn - sb);
                    const bool valid = lane < nb;
                    const uint32_t li = valid ? (uint32_t)list[qs + sb + lane] : 0u;
                    const uint32_t arr = c_arr[li], prm = c_prompt[li], ol = c_out[li];     // widened to 32 bits
                    const uint32_t ready = max(arr, rp.t_on);
                    const uint32_t prefill = rp.a + rp.b * prm;
                    const uint32_t tpot = rp.c + rp.d * ((prm + 1023u) >> 10);
                    const uint32_t dec = ol * tpot;
                    const uint32_t svc = prefill + dec;
                    // requests are in arrival order, so those arriving inside the window are a prefix
                    const uint32_t n_open = __popcll(__ballot(valid && ready < rp.t_off));
                    uint32_t start = ready;
                    uint32_t n_served = n_open;
                    if (n_open > 0u) {
                        const uint32_t ready0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)ready);
                        const unsigned long long idle = __ballot(S <= ready0);
                        const uint32_t n_idle = __popcll(idle);
                        // The first n_idle requests find a free slot whatever the earlier ones of the block
                        // did (a slot free at the first ready time stays free for them), so they start when
                        // ready and their finish times replace the idle slots' times in one permute.  It pays
                        // when that covers the whole block, or enough of it to be worth sorting afterwards.
                        uint32_t n_first = 0;
                        if (n_idle >= n_open || (in_order ? n_idle >= 16u : n_idle > 0u)) {
                            n_first = min(n_idle, n_open);
                            const uint32_t ri = __popcll(idle & lanes_below);
                            const uint32_t fin = ready + svc;
                            const uint32_t take = (uint32_t)__builtin_amdgcn_ds_bpermute((int)(ri << 2), (int)fin);
                            if (((idle >> lane) & 1ull) && ri < n_first) S = take;
                            in_order = false;
                        }
                        if (n_first < n_open) {
                            // the rest one by one, slot times sorted across the lanes
                            if (!in_order) S = wave_sort_ascending(S, lane);
                            in_order = true;
                            // The loop itself does not look at t_off.  Starts do not decrease along
                            // a queue, so the requests that would start at or after t_off are a
                            // suffix of the block: if there are any (at most once per replica, when
                            // its window closes), the slot times are put back and only the served
                            // prefix is run again.
                            // Start times are pushed into a vector from lane 0 (cheaper than writing
                            // lane j), so they come out in reverse order and are turned round after.
                            const uint32_t S_before = S;
                            uint32_t n_run = n_open;
                            for (;;) {
                                uint32_t pushed = 0;
                                auto step = [&](uint32_t j) {
                                    const uint32_t u = (uint32_t)__builtin_amdgcn_readfirstlane((int)S);
                                    const uint32_t st = max((uint32_t)__builtin_amdgcn_readlane((int)ready, (int)j), u);
                                    const uint32_t fj = st + (uint32_t)__builtin_amdgcn_readlane((int)svc, (int)j);
                                    S = min(wave_shift_down(S, kNever), max(S, fj));
                                    pushed = wave_shift_up(pushed, st);
                                };
                                uint32_t j = n_first;
                                for (; j + 2u <= n_run; j += 2u) {
                                    step(j);
                                    step(j + 1u);
                                }
                                if (j < n_run) step(j);
                                const uint32_t mine = (uint32_t)__builtin_amdgcn_ds_bpermute((int)((n_run - 1u - lane) << 2), (int)pushed);
                                if (lane >= n_first && lane < n_run) start = mine;
                                const uint32_t n_in_time = __popcll(__ballot(lane < n_run && start < rp.t_off));
                                if (n_in_time == n_run) break;
                                S = S_before;
                                n_run = n_in_time;      // not below n_first: those start when ready, before t_off
                            }
                            n_served = n_run;
                        }
                    }
                    if (lane < n_served) {
                        const uint32_t ttft = start - arr + prefill;
                        const uint32_t e2e = ttft + dec;
                        hist_add<kHist16>(hist, 0u, hist_bin_u32(ttft), 1u);
                        hist_add<kHist16>(hist, 1u, hist_bin_u32(tpot), 1u);
                        hist_add<kHist16>(hist, 2u, hist_bin_u32(e2e), 1u);
                        s_ttft += ttft;
                        s_e2e += e2e;
                        s_tpot += tpot;
                        last_fin = max(last_fin, start + svc);
                        n_ok += (ttft <= p.slo_ttft && tpot <= p.slo_tpot) ? 1u : 0u;
                    } else if (valid) {
                        n_rej += 1u;    // replica gone before the request could start
                    }
                }
                if (lane < B) slots[m * B + lane] = S;
                if (lane == 0) sorted[m] = in_order ? 1u : 0u;
            }
            }
            __syncthreads();
        }

        finish_candidate<kHist16>(p, hist, acc64, acc32, wtot, s_e2e, s_ttft, s_tpot, last_fin, n_ok, n_rej, &out[c]);
        __syncthreads();
    }
}

// ----------------------------------------------------------------------------------
// exact replay as three kernels: group -> replay -> reduce
// ----------------------------------------------------------------------------------
// The candidates of a batch are scored by three kernels that hand their intermediates over
// in a device scratch area sized once by ap_costmodel_set (the batch is cut so that the
// area stays within the last-level cache):
//   k_group_requests    per candidate and time chunk: replica histogram, scans, ballot-ranked
//                       stable scatter -> per-replica index lists (queue order = arrival order)
//   k_replay_queues     one LANE per (candidate, replica) queue; the B slot-free times of a
//                       queue are a binary min-heap in LDS (one column per lane, so lanes never
//                       collide on a bank); per request: start = max(ready, heap root), replace
//                       the root by the finish time, sift down.  64 queues advance per wavefront
//                       instruction, which is what makes saturated queues affordable.
//   k_reduce_candidates per candidate: LDS histograms of the per-request bins, p99s, sums.
// only_pending != 0 restricts all three to the candidates still marked pending.
struct QueuePartial {                  // what one queue contributes to its candidate's record
    unsigned long long sum_e2e, sum_ttft, sum_tpot;
    uint32_t last_fin, n_ok, n_rej, pad;
};

struct GroupParams {
    uint32_t R, M, chunk, n_chunks, key_bits;
    uint32_t qs_stride;                // uint16 entries per (candidate, chunk) in `qs`: M + 2, padded even
    uint16_t* qs;                      // [batch][n_chunks][qs_stride]: qs[m] = first list position of replica m
                                       //   in the chunk; qs[M] = number of listed requests; qs[M+1] unused
    uint16_t* list;                    // [batch][n_chunks * chunk] chunk-local request indices, by replica
    uint32_t* unknown;                 // [batch] requests naming no replica
};

constexpr uint32_t kGroupThreads = 512;
constexpr uint32_t kGroupWaves = kGroupThreads / kWave;
constexpr uint32_t kGroupMaxPerThread = 8;      // chunk <= 4096

__global__ __launch_bounds__(kGroupThreads) void k_group_requests(GroupParams p, const uint16_t* __restrict__ assign,
                                                                  const ap_metrics* __restrict__ out, uint32_t c0,
                                                                  uint32_t n_cand, uint32_t only_pending) {
    extern __shared__ __align__(16) unsigned char lds[];
    const uint32_t M = p.M, M1 = p.M + 1u;
    uint32_t* cnt = reinterpret_cast<uint32_t*>(lds);                    // [kGroupWaves][M+1]
    uint32_t* qstart = cnt + kGroupWaves * M1;                           // [M+2]
    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    const uint32_t w = wave_index();
    const uint32_t per_wave = p.chunk / kGroupWaves;                     // multiple of 64
    const uint32_t groups = per_wave / kWave;

    for (uint32_t cb = blockIdx.x; cb < n_cand; cb += gridDim.x) {
        const uint32_t c = c0 + cb;
        if (only_pending && !is_pending(out[c])) continue;
        const uint16_t* row = assign + (size_t)c * p.R;
        uint32_t n_unknown = 0;
        for (uint32_t j = 0; j < p.n_chunks; ++j) {
            const uint32_t r0 = j * p.chunk, n = min(p.chunk, p.R - r0);
            uint32_t key[kGroupMaxPerThread];
#pragma unroll
            for (uint32_t g = 0; g < kGroupMaxPerThread; ++g) {
                const uint32_t idx = w * per_wave + g * kWave + lane;
                key[g] = (g < groups && idx < n) ? min((uint32_t)__builtin_nontemporal_load(row + r0 + idx), M) : kNoKey;
            }
            for (uint32_t i = tid; i < kGroupWaves * M1; i += kGroupThreads) cnt[i] = 0u;
            __syncthreads();
            // (1) per-wavefront replica histogram
#pragma unroll
            for (uint32_t g = 0; g < kGroupMaxPerThread; ++g)
                if (key[g] != kNoKey) atomicAdd(&cnt[w * M1 + key[g]], 1u);
            __syncthreads();
            // (2) offsets: down the wavefronts per replica, then across replicas
            for (uint32_t m = tid; m <= M; m += kGroupThreads) {
                uint32_t run = 0;
                for (uint32_t ww = 0; ww < kGroupWaves; ++ww) {
                    const uint32_t t = cnt[ww * M1 + m];
                    cnt[ww * M1 + m] = run;
                    run += t;
                }
                qstart[m] = run;
            }
            __syncthreads();
            if (w == 0) {
                uint32_t carry = 0;
                for (uint32_t base = 0; base <= M; base += kWave) {
                    const uint32_t m = base + lane;
                    const uint32_t v = m <= M ? qstart[m] : 0u;
                    const uint32_t incl = wave_inclusive_scan(v, lane);
                    if (m <= M) qstart[m] = carry + incl - v;
                    carry += (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
                }
            }
            __syncthreads();
            // (3) stable scatter: rank among equal keys of a 64-request group by ballots
            uint16_t* lst = p.list + ((size_t)cb * p.n_chunks + j) * p.chunk;
#pragma unroll
            for (uint32_t g = 0; g < kGroupMaxPerThread; ++g) {
                if (g >= groups) break;
                const uint32_t k = key[g];
                uint32_t peers_lo, peers_hi;
                wave_peers(k, M, p.key_bits, peers_lo, peers_hi);
                if (k < M) {
                    const uint32_t rank = __builtin_amdgcn_mbcnt_hi(peers_hi, __builtin_amdgcn_mbcnt_lo(peers_lo, 0u));
                    const uint32_t total = __popc(peers_lo) + __popc(peers_hi);
                    const uint32_t base = qstart[k] + cnt[w * M1 + k];
                    lst[base + rank] = (uint16_t)(w * per_wave + g * kWave + lane);
                    if (rank + 1u == total) cnt[w * M1 + k] += total;
                } else if (k == M) {
                    n_unknown += 1u;
                }
            }
            uint16_t* qs = p.qs + ((size_t)cb * p.n_chunks + j) * p.qs_stride;
            for (uint32_t m = tid; m <= M; m += kGroupThreads) qs[m] = (uint16_t)qstart[m];
            __syncthreads();
        }
        n_unknown = wave_sum_u32(n_unknown);
        if (lane == 0 && n_unknown) atomicAdd(&p.unknown[cb], n_unknown);
    }
}

struct ReplayParams {
    const uint4* req;                  // [R] {arrival (relative us), prompt_len, out_len, 0}
    const DevReplica* rep;             // [M]
    const uint16_t* qs;
    const uint16_t* list;
    uint32_t* bins_te;                 // [batch][n_chunks * chunk] ttft bin | e2e bin << 16; 0xFFFFFFFF = rejected
    uint16_t* bins_p;                  // [batch][n_chunks * chunk] tpot bin
    QueuePartial* partial;             // [batch][M]
    uint32_t R, M, B, chunk, n_chunks, qs_stride;
    uint32_t slo_ttft, slo_tpot;
};

constexpr uint32_t kReplayWaves = 2;
constexpr uint32_t kReplayThreads = kReplayWaves * kWave;

__global__ __launch_bounds__(kReplayThreads) void k_replay_queues(ReplayParams p, const ap_metrics* __restrict__ out,
                                                                  uint32_t c0, uint32_t n_cand, uint32_t only_pending) {
    extern __shared__ __align__(16) unsigned char lds[];
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t w = wave_index();
    const uint32_t B = p.B, M = p.M;
    uint32_t* heap = reinterpret_cast<uint32_t*>(lds) + w * B * kWave + lane;      // node i of this lane: heap[i * 64]
    const uint32_t n_queues = n_cand * M;

    for (uint32_t q0 = (blockIdx.x * kReplayWaves + w) * kWave; q0 < n_queues; q0 += gridDim.x * kReplayThreads) {
        const uint32_t q = q0 + lane;
        const uint32_t cb = min(q, n_queues - 1u) / M, m = min(q, n_queues - 1u) % M;
        bool live = q < n_queues;
        if (live && only_pending && !is_pending(out[c0 + cb])) live = false;
        if (__ballot(live) == 0ull) continue;
        const DevReplica rp = p.rep[m];
        for (uint32_t i = 0; i < B; ++i) heap[i * kWave] = 0u;            // all slots free at time 0

        const uint16_t* qs = p.qs + (size_t)cb * p.n_chunks * p.qs_stride;
        const size_t cand_base = (size_t)cb * p.n_chunks * p.chunk;
        unsigned long long s_e2e = 0, s_ttft = 0, s_tpot = 0;
        uint32_t last_fin = 0, n_ok = 0, n_rej = 0;
        bool closed = false;                                              // the replica is gone for good
        uint32_t j = 0, k = 0, e = 0;
        if (live) { k = qs[m]; e = qs[m + 1]; }
        while (true) {
            // advance to the lane's next listed request (chunks in time order)
            while (live && k == e) {
                if (++j >= p.n_chunks) { live = false; break; }
                k = qs[j * p.qs_stride + m];
                e = qs[j * p.qs_stride + m + 1u];
            }
            if (__ballot(live) == 0ull) break;
            if (live) {
                const size_t pos = cand_base + (size_t)j * p.chunk + k;
                const uint32_t r = j * p.chunk + p.list[pos];
                ++k;
                const uint4 rq = p.req[r];
                const uint32_t ready = max(rq.x, rp.t_on);
                uint32_t te = 0xFFFFFFFFu, tp = 0xFFFFu;
                if (!closed) {
                    const uint32_t root = heap[0];
                    const uint32_t start = max(ready, root);
                    if (start >= rp.t_off) {
                        closed = true;            // starts never decrease along a queue: the rest is rejected too
                    } else {
                        const uint32_t prefill = rp.a + rp.b * rq.y;
                        const uint32_t tpot = rp.c + rp.d * ((rq.y + 1023u) >> 10);
                        const uint32_t dec = rq.z * tpot;
                        const uint32_t fin = start + prefill + dec;
                        // replace the root by `fin` and restore the heap order
                        uint32_t i = 0;
                        while (true) {
                            const uint32_t l = 2u * i + 1u;
                            if (l >= B) break;
                            const uint32_t cl = heap[l * kWave];
                            const uint32_t cr = l + 1u < B ? heap[(l + 1u) * kWave] : kNever;
                            const uint32_t cm = min(cl, cr);
                            if (fin <= cm) break;
                            heap[i * kWave] = cm;
                            i = cr < cl ? l + 1u : l;
                        }
                        heap[i * kWave] = fin;
                        const uint32_t ttft = start - rq.x + prefill;
                        const uint32_t e2e = ttft + dec;
                        te = hist_bin_u32(ttft) | (hist_bin_u32(e2e) << 16);
                        tp = hist_bin_u32(tpot);
                        s_ttft += ttft;
                        s_e2e += e2e;
                        s_tpot += tpot;
                        last_fin = max(last_fin, fin);
                        n_ok += (ttft <= p.slo_ttft && tpot <= p.slo_tpot) ? 1u : 0u;
                    }
                }
                if (closed) n_rej += 1u;
                p.bins_te[pos] = te;
                p.bins_p[pos] = (uint16_t)tp;
            }
        }
        if (q < n_queues && !(only_pending && !is_pending(out[c0 + cb]))) {
            QueuePartial qp;
            qp.sum_e2e = s_e2e; qp.sum_ttft = s_ttft; qp.sum_tpot = s_tpot;
            qp.last_fin = last_fin; qp.n_ok = n_ok; qp.n_rej = n_rej; qp.pad = 0u;
            p.partial[(size_t)cb * M + m] = qp;
        }
    }
}

struct ReduceParams {
    const uint16_t* qs;
    const uint32_t* bins_te;
    const uint16_t* bins_p;
    const QueuePartial* partial;
    uint32_t* unknown;                 // read, then cleared for the next batch
    uint32_t M, chunk, n_chunks, qs_stride;
};

template <bool kHist16>
__global__ __launch_bounds__(kThreads) void k_reduce_candidates(EvalParams p, ReduceParams rp, ap_metrics* out,
                                                                uint32_t c0, uint32_t n_cand, uint32_t only_pending) {
    extern __shared__ __align__(16) unsigned char lds[];
    uint32_t* hist = reinterpret_cast<uint32_t*>(lds);
    unsigned long long* acc64 = reinterpret_cast<unsigned long long*>(lds + p.off_misc);
    uint32_t* acc32 = reinterpret_cast<uint32_t*>(lds + p.off_misc + 24);
    uint32_t* wtot = reinterpret_cast<uint32_t*>(lds + p.off_misc + 64);
    const uint32_t tid = threadIdx.x;
    for (uint32_t cb = blockIdx.x; cb < n_cand; cb += gridDim.x) {
        const uint32_t c = c0 + cb;
        if (only_pending && !is_pending(out[c])) continue;
        hist_clear<kHist16>(hist);
        if (tid < 16u) reinterpret_cast<uint32_t*>(acc64)[tid] = 0u;
        __syncthreads();
        for (uint32_t j = 0; j < rp.n_chunks; ++j) {
            const uint32_t n_listed = rp.qs[((size_t)cb * rp.n_chunks + j) * rp.qs_stride + rp.M];
            const size_t base = ((size_t)cb * rp.n_chunks + j) * rp.chunk;
            for (uint32_t i = tid; i < n_listed; i += kThreads) {
                const uint32_t te = rp.bins_te[base + i];
                if (te != 0xFFFFFFFFu) {
                    hist_add<kHist16>(hist, 0u, te & 0xFFFFu, 1u);
                    hist_add<kHist16>(hist, 1u, rp.bins_p[base + i], 1u);
                    hist_add<kHist16>(hist, 2u, te >> 16, 1u);
                }
            }
        }
        unsigned long long s_e2e = 0, s_ttft = 0, s_tpot = 0;
        uint32_t last_fin = 0, n_ok = 0, n_rej = 0;
        for (uint32_t m = tid; m < rp.M; m += kThreads) {
            const QueuePartial qp = rp.partial[(size_t)cb * rp.M + m];
            s_e2e += qp.sum_e2e; s_ttft += qp.sum_ttft; s_tpot += qp.sum_tpot;
            last_fin = max(last_fin, qp.last_fin); n_ok += qp.n_ok; n_rej += qp.n_rej;
        }
        if (tid == 0) {
            n_rej += rp.unknown[cb];
            rp.unknown[cb] = 0u;
        }
        finish_candidate<kHist16>(p, hist, acc64, acc32, wtot, s_e2e, s_ttft, s_tpot, last_fin, n_ok, n_rej, &out[c]);
        __syncthreads();
    }
}

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

using EvalKernel = void (*)(EvalParams, const uint16_t*, ap_metrics*, uint32_t, uint32_t);

EvalKernel eval_kernel(bool hist16, bool len16) {
    if (hist16) return len16 ? k_eval_candidates<true, true> : k_eval_candidates<true, false>;
    return len16 ? k_eval_candidates<false, true> : k_eval_candidates<false, false>;
}


// ----------------------------------------------------------------------------------
// sparse candidates: children of one parent row, given as lists of (request, replica) edits
// ----------------------------------------------------------------------------------
// Children are small modifications of a parent (Section 5.4 "Synthesis Configuration",
// trade-off-aware mutation; Section 6.1 "Warm-start re-evolution": top candidates along with
// their mutations).  A child's row is the parent's with its edits applied front to back; a later
// edit of a request replaces an earlier one and an edit naming a request >= R changes nothing.
//
// With identical, always-available replicas the parent is analysed once (k_parent_occupancy):
// peak[m] is the largest number of the parent's requests replica m has in service at the same
// moment when nobody waits, i.e. the depth of the intervals [arrival, arrival + service).  A
// child's requests on replica m are a subset of the parent's there plus the requests its edits
// send to m, so their depth is at most peak[m] + (edits naming m).  Where that stays within B for
// every replica no request of the child ever finds the B slots taken, nobody waits, and the
// child's record is the nominal one - decided from the edit list alone, without its row.  Every
// other child gets its row written out and goes through the dense path (screening, then replay).
struct ChildParams {
    const uint16_t* parent;       // [R]
    const uint32_t* room;         // [M] B - peak[m], or 0 where the parent already exceeds B
    const ap_metrics* nominal;
    uint16_t* rows;               // [max_children][R] rows of the children the dense path has to look at
    uint32_t R, M, key_bits;      // key_bits: bits of R - 1
    uint32_t certify;             // 0: no shortcut (replicas differ, windows, parent not contention-free): rows for all
};

constexpr uint32_t kChildWaves = 4;
constexpr uint32_t kChildThreads = kChildWaves * kWave;
constexpr uint32_t kOccupancyThreads = 256;
constexpr uint32_t kOccupancyWaves = kOccupancyThreads / kWave;
constexpr uint32_t kOccupancyPerThread = 16;      // parent ids per thread and step
constexpr uint32_t kOccupancyStep = kOccupancyThreads * kOccupancyPerThread;

// One workgroup per replica walks the parent row in steps of 4096 ids.  All its threads pick out
// the replica's requests of the step (each thread 16 consecutive ids; counts scanned across the
// workgroup; request indices written to an LDS list in arrival order), then the first wavefront
// takes the list through the queue-free schedule: lane l holds the finish time of the request
// that last used "slot" l, a request takes the lowest lane that is free at its arrival (finish
// <= arrival), and the number of busy lanes plus one is the depth at that moment.  More than 64
// at once is reported as 65 (B never exceeds 64).  peak[M] counts the parent's requests that
// name no replica of the table.
__global__ __launch_bounds__(kOccupancyThreads) void k_parent_occupancy(EvalParams p, const uint16_t* __restrict__ parent,
                                                                        uint32_t* __restrict__ peak,
                                                                        uint32_t* __restrict__ room) {
    __shared__ uint32_t list[kOccupancyStep];     // requests of this replica in the current step
    __shared__ uint32_t wave_total[kOccupancyWaves];
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wv = wave_index(), m = blockIdx.x;
    const DevReplica rp = p.rep[0];
    uint32_t slot_finish = 0u, deepest = 0u, unknown = 0u;
    // my 16 ids of a step: two 16-byte loads where the row has them all (the parent buffer is 16-byte
    // aligned and a thread's run starts at a multiple of 16 ids), one by one at the ragged end
    auto fetch = [&](uint4 (&into)[2], uint32_t r0) {
        const uint32_t at = r0 + tid * kOccupancyPerThread;
        if (at + kOccupancyPerThread <= p.R) {
            into[0] = reinterpret_cast<const uint4*>(parent + at)[0];
            into[1] = reinterpret_cast<const uint4*>(parent + at)[1];
        } else {
            uint32_t w[8];
#pragma unroll
            for (uint32_t k = 0; k < 8u; ++k) {
                const uint32_t lo = at + 2u * k < p.R ? (uint32_t)parent[at + 2u * k] : 0xFFFFu;
                const uint32_t hi = at + 2u * k + 1u < p.R ? (uint32_t)parent[at + 2u * k + 1u] : 0xFFFFu;
                w[k] = lo | (hi << 16);
            }
            into[0] = make_uint4(w[0], w[1], w[2], w[3]);
            into[1] = make_uint4(w[4], w[5], w[6], w[7]);
        }
    };
    uint4 ids_next[2];
    fetch(ids_next, 0u);
    for (uint32_t r0 = 0; r0 < p.R; r0 += kOccupancyStep) {
        // as a bit mask: which of my 16 ids name this replica (absent ones read as 0xFFFF and are skipped below)
        const uint32_t mine = r0 + tid * kOccupancyPerThread;
        const uint32_t w[8] = {ids_next[0].x, ids_next[0].y, ids_next[0].z, ids_next[0].w,
                               ids_next[1].x, ids_next[1].y, ids_next[1].z, ids_next[1].w};
        if (r0 + kOccupancyStep < p.R) fetch(ids_next, r0 + kOccupancyStep);   // in flight during the rest of this step
        uint32_t hits = 0u;
#pragma unroll
        for (uint32_t k = 0; k < kOccupancyPerThread; ++k) {
            const uint32_t id = (w[k >> 1] >> ((k & 1u) << 4)) & 0xFFFFu;
            const bool present = mine + k < p.R;
            hits |= (present && id == m ? 1u : 0u) << k;
            unknown += (present && id >= p.M) ? 1u : 0u;
        }
        const uint32_t n_mine = (uint32_t)__popc(hits);
        const uint32_t upto = wave_inclusive_scan(n_mine, lane);
        if (lane == 63u) wave_total[wv] = upto;
        __syncthreads();
        uint32_t before = upto - n_mine, n_list = 0u;
#pragma unroll
        for (uint32_t j = 0; j < kOccupancyWaves; ++j) {
            before += j < wv ? wave_total[j] : 0u;
            n_list += wave_total[j];
        }
        for (uint32_t h = hits; h != 0u; h &= h - 1u) list[before++] = mine + (uint32_t)__ffs((int)h) - 1u;
        __syncthreads();
        if (wv == 0u) {
            for (uint32_t i0 = 0; i0 < n_list; i0 += kWave) {
                uint32_t arrival = 0u, finish = 0u;
                if (i0 + lane < n_list) {
                    const uint32_t r = list[i0 + lane];
                    const uint32_t prm = p.prompt[r];
                    arrival = p.arrival[r];
                    finish = arrival + rp.a + rp.b * prm + p.outlen[r] * (rp.c + rp.d * ((prm + 1023u) >> 10));
                }
                const uint32_t n_here = min(kWave, n_list - i0);
                for (uint32_t k = 0; k < n_here; ++k) {
                    const uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int)arrival, (int)k);
                    const uint32_t f = (uint32_t)__builtin_amdgcn_readlane((int)finish, (int)k);
                    const unsigned long long busy = __ballot(slot_finish > a);
                    deepest = max(deepest, (uint32_t)__popcll(busy) + 1u);
                    if (~busy != 0ull && lane == (uint32_t)__ffsll((long long)~busy) - 1u) slot_finish = f;
                }
            }
        }
        // the next step's scan may overwrite wave_total and list only after everyone is done with them
        __syncthreads();
    }
    if (tid == 0u) {
        peak[m] = deepest;
        room[m] = deepest <= p.B ? p.B - deepest : 0u;
    }
    if (m == 0u) {
        unknown = wave_sum_u32(unknown);
        if (lane == 0u) wave_total[wv] = unknown;
        __syncthreads();
        if (tid == 0u) {
            uint32_t total = 0u;
            for (uint32_t j = 0; j < kOccupancyWaves; ++j) total += wave_total[j];
            peak[p.M] = total;
        }
    }
}

// One wavefront per child.  certify: count the child's edits per replica in LDS and compare with
// the room the parent leaves; a child that passes gets the nominal record.  A child that does not
// pass (too many edits for some replica, or an edit naming a replica outside the table) gets the
// pending mark and its row: the parent's, then its edits in batches of 64, the lanes of a batch
// that name the same request settled in favour of the highest lane, batches in list order.
__global__ __launch_bounds__(kChildThreads) void k_certify_children(ChildParams p, const uint32_t* __restrict__ first,
                                                                    const uint32_t* __restrict__ request,
                                                                    const uint16_t* __restrict__ replica,
                                                                    ap_metrics* __restrict__ out, uint32_t C) {
    extern __shared__ __align__(16) unsigned char lds[];
    const uint32_t lane = threadIdx.x & 63u, w = wave_index();
    uint32_t* count = reinterpret_cast<uint32_t*>(lds) + w * p.M;            // this wavefront's: edits per replica
    uint32_t* room = reinterpret_cast<uint32_t*>(lds) + kChildWaves * p.M;   // the workgroup's copy of p.room
    for (uint32_t m = lane; m < p.M; m += kWave) count[m] = 0u;
    unsigned long long nominal_word = 0ull;                                  // lanes 0..7: the record of a child that passes
    if (p.certify != 0u) {
        for (uint32_t m = threadIdx.x; m < p.M; m += kChildThreads) room[m] = p.room[m];
        if (lane < 8u) nominal_word = reinterpret_cast<const unsigned long long*>(p.nominal)[lane];
    }
    __syncthreads();
    for (uint32_t c = blockIdx.x * kChildWaves + w; c < C; c += gridDim.x * kChildWaves) {
        const unsigned long long e0 = first[c], e1 = first[c + 1u];          // empty or reversed: no edits
        bool dense = p.certify == 0u;
        if (!dense) {
            bool fail = false;
            // rounds of kInFlight loads of both arrays per lane; the next round is requested before the
            // current one is counted, so the lists stream in without a pause between rounds
            constexpr uint32_t kInFlight = 8;
            uint32_t r[kInFlight], m[kInFlight], r_next[kInFlight], m_next[kInFlight];
            auto fetch = [&](uint32_t (&rq)[kInFlight], uint32_t (&rp)[kInFlight], unsigned long long b) {
#pragma unroll
                for (uint32_t k = 0; k < kInFlight; ++k) {
                    const unsigned long long e = b + k * kWave + lane;
                    rq[k] = e < e1 ? request[e] : kNoKey;                    // past the end: names no request
                    rp[k] = e < e1 ? (uint32_t)replica[e] : 0u;
                }
            };
            if (e0 < e1) fetch(r_next, m_next, e0);
            for (unsigned long long b = e0; b < e1; b += kInFlight * kWave) {
#pragma unroll
                for (uint32_t k = 0; k < kInFlight; ++k) {
                    r[k] = r_next[k];
                    m[k] = m_next[k];
                }
                if (b + kInFlight * kWave < e1) fetch(r_next, m_next, b + kInFlight * kWave);
#pragma unroll
                for (uint32_t k = 0; k < kInFlight; ++k) {
                    if (r[k] < p.R) {
                        if (m[k] < p.M) atomicAdd(&count[m[k]], 1u);
                        else fail = true;
                    }
                }
            }
            for (uint32_t m = lane; m < p.M; m += kWave) {
                fail = fail || count[m] > room[m];
                count[m] = 0u;
            }
            dense = __ballot(fail) != 0ull;
            if (lane < 8u) reinterpret_cast<unsigned long long*>(&out[c])[lane] = dense ? ~0ull : nominal_word;
        }
        if (!dense) continue;
        uint16_t* row = p.rows + (size_t)c * p.R;
        if (p.R % 8u == 0u) {                                                // rows are then 16-byte aligned
            const uint4* src = reinterpret_cast<const uint4*>(p.parent);
            uint4* dst = reinterpret_cast<uint4*>(row);
            for (uint32_t i = lane; i < p.R / 8u; i += kWave) dst[i] = src[i];
        } else {
            for (uint32_t i = lane; i < p.R; i += kWave) row[i] = p.parent[i];
        }
        for (unsigned long long b = e0; b < e1; b += kWave) {
            __threadfence();                                                 // the copy, or the batch before, has landed
            const unsigned long long e = b + lane;
            const uint32_t r = e < e1 ? request[e] : kNoKey;
            const uint16_t m = e < e1 ? replica[e] : (uint16_t)0;
            uint32_t lo, hi;
            wave_peers(r, p.R, p.key_bits, lo, hi);                          // lanes of this batch naming my request
            const unsigned long long peers = ((unsigned long long)hi << 32) | lo;
            if (e < e1 && r < p.R && ((peers >> lane) >> 1) == 0ull) row[r] = m;
        }
    }
}

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
    uint32_t* d_span = nullptr;       // [R] contention-free service intervals in ticks, valid when screen is set
    uint32_t* d_span_t = nullptr;     // the same, lane-major for the one-wavefront screening kernel
    uint32_t* d_pair = nullptr;       // one word per two requests (eight-wavefront screening kernel, when it fits)
    bool screen_packed = false;       // that kernel reads d_pair instead of d_span
    ap_metrics* d_nominal = nullptr;  // record shared by all contention-free candidates
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
    uint16_t* d_rows = nullptr;       // [max_children][R]
    size_t rows_bytes = 0;
    uint32_t max_children = 0;
    bool has_parent = false;
    ChildParams child_params{};
};

// The dense path on C rows: screening where it applies, then the exact replay of what is left.
// marked: only rows whose record carries the pending mark are looked at (screening applies).
static ap_status launch_dense(const ap_workload* w, const uint16_t* d_assign, uint32_t C, ap_metrics* d_out,
                              hipStream_t stream, bool marked) {
    if (w->screen) {
        const uint32_t blocks = std::min((C + kScreenWaves - 1u) / kScreenWaves, w->n_cu * 64u);
        // rows start on 4-byte boundaries when R is even and the batch itself does
        const bool aligned = (w->R % 2u == 0u) && (reinterpret_cast<uintptr_t>(d_assign) % 4u == 0u);
        typedef void (*screen_fn)(ScreenParams, const uint16_t*, ap_metrics*, uint32_t);
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
                               dim3(kWideThreads), w->screen_wide_lds_bytes, stream, w->screen_params, d_assign, d_out, C);
        } else {
            static const screen_fn narrow[4] = {k_screen_candidates<false, false>, k_screen_candidates<true, false>,
                                                k_screen_candidates<false, true>, k_screen_candidates<true, true>};
            const uint32_t grid = marked ? std::max((C + kScreenThreads - 1u) / kScreenThreads, std::min(blocks, w->n_cu * 8u))
                                         : blocks;
            hipLaunchKernelGGL(narrow[(aligned ? 1 : 0) + (marked ? 2 : 0)], dim3(grid), dim3(kScreenThreads),
                               w->screen_lds_bytes, stream, w->screen_params, d_assign, d_out, C);
        }
        if (hipGetLastError() != hipSuccess) return AP_ERR_DEVICE;
    }
    const uint32_t pending_only = w->screen ? 1u : 0u;
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
        if (hipGetLastError() != hipSuccess) return AP_ERR_DEVICE;
        return AP_OK;
    }
    // After screening, most workgroups only find out that nothing is left for them: as many as can be
    // resident at once look at all the records together.
    const uint32_t grid = std::min(C, pending_only ? w->resident_grid : w->max_grid);
    hipLaunchKernelGGL(eval_kernel(w->hist16, w->len16), dim3(grid), dim3(kThreads), w->lds_bytes, stream, w->params,
                       d_assign, d_out, C, pending_only);
    if (hipGetLastError() != hipSuccess) return AP_ERR_DEVICE;
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
                        hipMalloc(&w->d_nominal, sizeof(ap_metrics)) != hipSuccess))
        st = AP_ERR_ALLOC;
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

ap_status ap_costmodel_set(ap_workload* w, const ap_replica* replicas, uint32_t M, uint32_t B, const ap_slo* slo) {
    if (!w || !replicas || !slo || M == 0 || B == 0) return AP_ERR_INVALID;
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
    // distinct coefficient sets
    std::vector<const ap_replica*> kinds;
    for (uint32_t m = 0; m < M; ++m) {
        bool seen = false;
        for (const ap_replica* k : kinds)
            seen = seen || (k->prefill_base_us == replicas[m].prefill_base_us &&
                            k->prefill_per_tok_us == replicas[m].prefill_per_tok_us &&
                            k->decode_base_us == replicas[m].decode_base_us &&
                            k->decode_per_kctx_us == replicas[m].decode_per_kctx_us);
        if (!seen) kinds.push_back(&replicas[m]);
    }
    uint64_t total = latest;
    uint64_t latest_unqueued = 0;      // latest finish if nobody ever waited (arrival + service)
    uint64_t longest_pair = 0;         // longest time from the arrival of request 2q to the unqueued finish of 2q or 2q+1
    uint64_t service_sum = 0;
    for (uint32_t r = 0; r < w->R; ++r) {
        const uint64_t prompt = (uint64_t)w->h_prompt[r], outl = (uint64_t)w->h_out[r];
        uint64_t worst = 0;
        for (const ap_replica* k : kinds) {
            // each term stays far below 2^64: coefficients < 2^32, lengths < 2^31
            uint64_t prefill = (uint64_t)k->prefill_base_us + (uint64_t)k->prefill_per_tok_us * prompt;
            uint64_t tpot = (uint64_t)k->decode_base_us + (uint64_t)k->decode_per_kctx_us * ((prompt + 1023u) >> 10);
            if (tpot > limit || prefill > limit) return AP_ERR_RANGE;
            uint64_t svc = prefill + outl * tpot;
            worst = std::max(worst, svc);
        }
        total += worst;
        service_sum += worst;
        latest_unqueued = std::max<uint64_t>(latest_unqueued, (uint64_t)w->h_arrival[r] + worst);
        longest_pair = std::max<uint64_t>(longest_pair, (uint64_t)w->h_arrival[r] + worst - w->h_arrival[r & ~1u]);
        if (total > limit) return AP_ERR_RANGE;
    }

    // ---- LDS plan: the largest chunk that fits ------------------------------------------
    if (hipSetDevice(w->device) != hipSuccess) return AP_ERR_DEVICE;
    int lds_cap = 0, n_cu = 0;
    if (hipDeviceGetAttribute(&lds_cap, hipDeviceAttributeMaxSharedMemoryPerBlock, w->device) != hipSuccess ||
        hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, w->device) != hipSuccess)
        return AP_ERR_DEVICE;
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
        if (hipFuncGetAttributes(&attr, reinterpret_cast<const void*>(eval_kernel(hist16, w->len16))) != hipSuccess)
            return AP_ERR_DEVICE;
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
        d.a = rp.prefill_base_us;
        d.b = rp.prefill_per_tok_us;
        d.c = rp.decode_base_us;
        d.d = rp.decode_per_kctx_us;
        if (rp.t_on_us >= rp.t_off_us || rp.t_off_us <= w->base_us) {
            d.t_on = 0;      // the window is empty or closed before the trace: nothing is ever served
            d.t_off = 0;
        } else {
            d.t_on = rp.t_on_us <= w->base_us ? 0u : (uint32_t)(rp.t_on_us - w->base_us);
            d.t_off = (uint32_t)std::min<uint64_t>(rp.t_off_us - w->base_us, kNever);
        }
    }
    if (hipMemcpy(w->d_rep, dev.data(), sizeof(DevReplica) * M, hipMemcpyHostToDevice) != hipSuccess ||
        (!use_pipeline && hipFuncSetAttribute(reinterpret_cast<const void*>(eval_kernel(hist16, w->len16)),
                                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess) ||
        hipFuncSetAttribute(hist16 ? reinterpret_cast<const void*>(&k_nominal_metrics<true>)
                                   : reinterpret_cast<const void*>(&k_nominal_metrics<false>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)reduce_lds) != hipSuccess) {
        (void)hipGetLastError();
        w->has_model = false;     // the replica table on the device may be half-written
        return AP_ERR_DEVICE;
    }

    p.arrival = w->d_arrival;
    p.prompt = w->d_prompt;
    p.outlen = w->d_out;
    p.rep = w->d_rep;
    p.R = w->R;
    p.key_bits = 0;
    while (((M - 1u) >> p.key_bits) != 0u) ++p.key_bits;       // bits needed for the replica ids 0..M-1
    p.slo_ttft = (uint32_t)std::min<uint64_t>(slo->ttft_us, kNever);
    p.slo_tpot = (uint32_t)std::min<uint64_t>(slo->tpot_us, kNever);
    p.penalty = slo->penalty_us;
    p.penalty_bin = ap_hist_bin(slo->penalty_us);
    p.k99 = (uint32_t)((99ull * w->R + 99ull) / 100ull);
    w->has_model = false;
    w->has_parent = false;    // its analysis belonged to the previous cost model
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
            if (w->d_scratch && hipFree(w->d_scratch) != hipSuccess) return AP_ERR_DEVICE;
            w->d_scratch = nullptr;
            w->scratch_bytes = 0;
            if (hipMalloc(&w->d_scratch, off) != hipSuccess) {
                (void)hipGetLastError();
                return AP_ERR_ALLOC;
            }
            w->scratch_bytes = off;
        }
        if (hipMemset(w->d_scratch + o_unk, 0, (size_t)batch * 4u) != hipSuccess) return AP_ERR_DEVICE;
        w->batch = batch;
        GroupParams gp{};
        gp.R = R; gp.M = M; gp.chunk = chunk_g; gp.n_chunks = n_chunks; gp.key_bits = p.key_bits; gp.qs_stride = qs_stride;
        gp.qs = reinterpret_cast<uint16_t*>(w->d_scratch + o_qs);
        gp.list = reinterpret_cast<uint16_t*>(w->d_scratch + o_list);
        gp.unknown = reinterpret_cast<uint32_t*>(w->d_scratch + o_unk);
        w->group_params = gp;
        w->group_lds_bytes = (kGroupWaves * (M + 1u) + M + 2u) * 4u;
        ReplayParams qp{};
        qp.req = w->d_req; qp.rep = w->d_rep; qp.qs = gp.qs; qp.list = gp.list;
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
            return AP_ERR_DEVICE;
    }

    // ---- screening plan: only for identical replicas that are available throughout ------
    bool always_on = true;
    for (const DevReplica& d : dev) always_on = always_on && d.t_on == 0u && d.t_off == kNever;
    w->screen = always_on && kinds.size() == 1;
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
        hipLaunchKernelGGL(hist16 ? k_nominal_metrics<true> : k_nominal_metrics<false>, dim3(1), dim3(kThreads),
                           reduce_lds, nullptr, w->reduce_eval, w->d_span, w->d_span_t,
                           w->screen_packed ? w->d_pair : nullptr, (uint32_t)tick_us, w->d_nominal);
        if (hipGetLastError() != hipSuccess || hipDeviceSynchronize() != hipSuccess) {
            (void)hipGetLastError();
            return AP_ERR_DEVICE;
        }
    }
    w->has_model = true;
    return AP_OK;
}

ap_status ap_eval_candidates(const ap_workload* w, const uint16_t* d_assign, uint32_t C, ap_metrics* d_out,
                             void* hip_stream) {
    if (!w) return AP_ERR_INVALID;
    if (!w->has_model) return AP_ERR_STATE;
    if (C == 0) return AP_OK;
    if (!d_assign || !d_out) return AP_ERR_INVALID;
    return launch_dense(w, d_assign, C, d_out, static_cast<hipStream_t>(hip_stream), false);
}

ap_status ap_parent_set(ap_workload* w, const uint16_t* parent, uint32_t max_children) {
    if (!w || !parent || max_children == 0) return AP_ERR_INVALID;
    if (!w->has_model) return AP_ERR_STATE;
    if (hipSetDevice(w->device) != hipSuccess) return AP_ERR_DEVICE;
    w->has_parent = false;
    if ((uint64_t)max_children > (UINT64_MAX / sizeof(uint16_t)) / w->R) return AP_ERR_ALLOC;     // the rows cannot exist
    const size_t need = (size_t)max_children * w->R * sizeof(uint16_t);
    if ((!w->d_parent && hipMalloc(&w->d_parent, (size_t)w->R * sizeof(uint16_t)) != hipSuccess) ||
        (!w->d_peak && hipMalloc(&w->d_peak, sizeof(uint32_t) * (AP_MAX_REPLICAS + 1u)) != hipSuccess) ||
        (!w->d_room && hipMalloc(&w->d_room, sizeof(uint32_t) * AP_MAX_REPLICAS) != hipSuccess)) {
        (void)hipGetLastError();
        return AP_ERR_ALLOC;
    }
    if (need > w->rows_bytes) {
        if (w->d_rows && hipFree(w->d_rows) != hipSuccess) return AP_ERR_DEVICE;
        w->d_rows = nullptr;
        w->rows_bytes = 0;
        if (hipMalloc(&w->d_rows, need) != hipSuccess) {
            (void)hipGetLastError();
            return AP_ERR_ALLOC;
        }
        w->rows_bytes = need;
    }
    if (hipMemcpy(w->d_parent, parent, (size_t)w->R * sizeof(uint16_t), hipMemcpyHostToDevice) != hipSuccess)
        return AP_ERR_DEVICE;
    const uint32_t M = w->params.M;
    bool certify = false;
    if (w->screen) {
        // the shortcut needs the nominal record, i.e. identical replicas that are always available
        hipLaunchKernelGGL(k_parent_occupancy, dim3(M), dim3(kOccupancyThreads), 0, nullptr, w->params, w->d_parent, w->d_peak,
                           w->d_room);
        std::vector<uint32_t> peak(M + 1u);
        if (hipGetLastError() != hipSuccess ||
            hipMemcpy(peak.data(), w->d_peak, sizeof(uint32_t) * (M + 1u), hipMemcpyDeviceToHost) != hipSuccess) {
            (void)hipGetLastError();
            return AP_ERR_DEVICE;
        }
        // ... and a parent that is contention-free itself and names only replicas of the table
        certify = peak[M] == 0u;
        for (uint32_t m = 0; m < M; ++m) certify = certify && peak[m] <= w->params.B;
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
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const uint32_t blocks = std::min((C + kChildWaves - 1u) / kChildWaves, w->n_cu * 64u);
    hipLaunchKernelGGL(k_certify_children, dim3(blocks), dim3(kChildThreads), (kChildWaves + 1u) * w->child_params.M * 4u, stream,
                       w->child_params, d_edit_first, d_edit_request, d_edit_replica, d_out, C);
    if (hipGetLastError() != hipSuccess) return AP_ERR_DEVICE;
    return launch_dense(w, w->d_rows, C, d_out, stream, w->child_params.certify != 0u);
}

ap_status ap_workload_destroy(ap_workload* w) {
    if (!w) return AP_OK;
    bool ok = true;
    if (w->d_arrival) ok = (hipFree(w->d_arrival) == hipSuccess) && ok;
    if (w->d_prompt) ok = (hipFree(w->d_prompt) == hipSuccess) && ok;
    if (w->d_out) ok = (hipFree(w->d_out) == hipSuccess) && ok;
    if (w->d_rep) ok = (hipFree(w->d_rep) == hipSuccess) && ok;
    if (w->d_req) ok = (hipFree(w->d_req) == hipSuccess) && ok;
    if (w->d_scratch) ok = (hipFree(w->d_scratch) == hipSuccess) && ok;
    if (w->d_span) ok = (hipFree(w->d_span) == hipSuccess) && ok;
    if (w->d_span_t) ok = (hipFree(w->d_span_t) == hipSuccess) && ok;
    if (w->d_pair) ok = (hipFree(w->d_pair) == hipSuccess) && ok;
    if (w->d_nominal) ok = (hipFree(w->d_nominal) == hipSuccess) && ok;
    if (w->d_parent) ok = (hipFree(w->d_parent) == hipSuccess) && ok;
    if (w->d_peak) ok = (hipFree(w->d_peak) == hipSuccess) && ok;
    if (w->d_room) ok = (hipFree(w->d_room) == hipSuccess) && ok;
    if (w->d_rows) ok = (hipFree(w->d_rows) == hipSuccess) && ok;
    delete w;
    return ok ? AP_OK : AP_ERR_DEVICE;
}

}  // extern "C"
