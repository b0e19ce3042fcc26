// Constants, kernel parameter blocks and wavefront / histogram helpers shared by all kernels.
#ifndef AP_COMMON_HPP
#define AP_COMMON_HPP

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
    uint32_t a, b, c, d;      // cost coefficients; with cost tables: a = first entry of the replica's type (type * R)
    uint32_t t_on, t_off;     // window, relative microseconds (t_off == kNever: never leaves)
};

struct EvalParams {
    const uint32_t* arrival;  // [R] relative microseconds
    const uint32_t* prompt;   // [R]
    const uint32_t* outlen;   // [R]
    const DevReplica* rep;    // [M]
    const uint32_t* tab_prefill;  // [T][R] microseconds of prefill per replica type and request, or null:
    const uint32_t* tab_tpot;     // [T][R] microseconds per output token       the linear stand-in applies
    uint32_t R, M, B, chunk, key_bits;
    uint32_t slo_ttft, slo_tpot;
    uint32_t penalty_bin, k99;
    uint64_t penalty;
    uint32_t* replayed;       // device counter: candidates that went through the exact replay kernels
    // byte offsets into dynamic LDS
    uint32_t off_slots, off_sorted, off_close, off_cnt, off_qstart, off_list, off_arr, off_prompt, off_out, off_misc;
};

// Prefill time and time per output token of request r (prompt length `prompt`) on a replica:
// the linear stand-in for the serve-latency equation, or the caller's tables (any cost model
// evaluated beforehand, e.g. the roofline sums of Appendix "Serving Simulator").
template <bool kTabled>
__device__ __forceinline__ void request_cost(const uint32_t* __restrict__ tab_prefill, const uint32_t* __restrict__ tab_tpot,
                                             const DevReplica& rp, uint32_t r, uint32_t prompt, uint32_t& prefill,
                                             uint32_t& tpot) {
    if (kTabled) {
        prefill = tab_prefill[rp.a + r];
        tpot = tab_tpot[rp.a + r];
    } else {
        prefill = rp.a + rp.b * prompt;
        tpot = rp.c + rp.d * ((prompt + 1023u) >> 10);
    }
}
__device__ __forceinline__ void request_cost(const uint32_t* tab_prefill, const uint32_t* tab_tpot, const DevReplica& rp,
                                             uint32_t r, uint32_t prompt, uint32_t& prefill, uint32_t& tpot) {
    if (tab_prefill != nullptr) request_cost<true>(tab_prefill, tab_tpot, rp, r, prompt, prefill, tpot);
    else request_cost<false>(tab_prefill, tab_tpot, rp, r, prompt, prefill, tpot);
}

// ----------------------------------------------------------------------------------
// wavefront helpers (64 lanes)
// ----------------------------------------------------------------------------------
// Index of this wavefront in its workgroup, as a wave-uniform (scalar) value: loops and
// table lookups that depend on it then stay on the scalar unit.
__device__ __forceinline__ uint32_t wave_index() {
    return (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
}

// Inclusive prefix sum over the lanes on the vector ALU's cross-lane path: a scan inside each row of 16
// lanes (the row shifted right by 1, 2, 4, 8; a lane without a source adds nothing), then the last lane
// of rows 0 and 2 added to rows 1 and 3, then lane 31 added to rows 2 and 3.
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v, uint32_t /*lane*/) {
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111 /* row_shr:1 */, 0xF, 0xF, false);
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112 /* row_shr:2 */, 0xF, 0xF, false);
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114 /* row_shr:4 */, 0xF, 0xF, false);
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118 /* row_shr:8 */, 0xF, 0xF, false);
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142 /* row_bcast:15 */, 0xA, 0xF, false);
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143 /* row_bcast:31 */, 0xC, 0xF, false);
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

// The value of lane (i ^ J) for every lane i.  J = 1, 2: a permutation inside each group of four lanes;
// J = 4, 8: the row of 16 lanes shifted left for the lanes whose bit J is clear and right for the
// others (two moves into one register, each writing the groups of four lanes it is meant for) - all on
// the vector ALU's cross-lane path.  J = 16, 32 cross rows and take the shuffle through the LDS crossbar.
template <uint32_t J>
__device__ __forceinline__ uint32_t lane_xor(uint32_t v) {
    if (J == 1u) return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0xB1 /* quad_perm:[1,0,3,2] */, 0xF, 0xF, false);
    if (J == 2u) return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x4E /* quad_perm:[2,3,0,1] */, 0xF, 0xF, false);
    if (J == 4u) {
        const int t = __builtin_amdgcn_update_dpp((int)v, (int)v, 0x104 /* row_shl:4 */, 0xF, 0x5, false);
        return (uint32_t)__builtin_amdgcn_update_dpp(t, (int)v, 0x114 /* row_shr:4 */, 0xF, 0xA, false);
    }
    if (J == 8u) {
        const int t = __builtin_amdgcn_update_dpp((int)v, (int)v, 0x108 /* row_shl:8 */, 0xF, 0x3, false);
        return (uint32_t)__builtin_amdgcn_update_dpp(t, (int)v, 0x118 /* row_shr:8 */, 0xF, 0xC, false);
    }
    return (uint32_t)__shfl_xor((int)v, (int)J);
}

// Ascending bitonic sort of one value per lane across the wavefront.
template <uint32_t K, uint32_t J>
__device__ __forceinline__ uint32_t wave_sort_step(uint32_t v, uint32_t lane) {
    const uint32_t other = lane_xor<J>(v);
    const bool keep_min = ((lane & J) == 0u) == ((lane & K) == 0u);
    return keep_min ? min(v, other) : max(v, other);
}
template <uint32_t K>
__device__ __forceinline__ uint32_t wave_sort_merge(uint32_t v, uint32_t lane) {
    if (K >= 64u) v = wave_sort_step<K, 32u>(v, lane);
    if (K >= 32u) v = wave_sort_step<K, 16u>(v, lane);
    if (K >= 16u) v = wave_sort_step<K, 8u>(v, lane);
    if (K >= 8u) v = wave_sort_step<K, 4u>(v, lane);
    if (K >= 4u) v = wave_sort_step<K, 2u>(v, lane);
    return wave_sort_step<K, 1u>(v, lane);
}
__device__ __forceinline__ uint32_t wave_sort_ascending(uint32_t v, uint32_t lane) {
    v = wave_sort_merge<2u>(v, lane);
    v = wave_sort_merge<4u>(v, lane);
    v = wave_sort_merge<8u>(v, lane);
    v = wave_sort_merge<16u>(v, lane);
    v = wave_sort_merge<32u>(v, lane);
    return wave_sort_merge<64u>(v, lane);
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

}  // namespace

#endif  // AP_COMMON_HPP
