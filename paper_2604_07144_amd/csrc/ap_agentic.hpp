// Agentic workflows on a disaggregated prefill/decode cluster: one wavefront replays one candidate plan.
#ifndef AP_AGENTIC_HPP
#define AP_AGENTIC_HPP

#include "ap_common.hpp"

namespace {

// ----------------------------------------------------------------------------------
// candidate plans for multi-call workflows (Section 8.3; Appendix, Formulation for Agentic Request)
// ----------------------------------------------------------------------------------
// A call is released when its workflow has arrived and all its predecessors have completed; it is
// prefilled on its prefill instance (one call at a time, the waiting call with the smallest
// (key, index) first), then decoded on its decode instance, which admits its first waiting call as
// soon as the call's in + out tokens fit the free part of the instance's token budget (no
// overtaking).  Events of one instant are applied as decode completions, prefill completions,
// releases, decode admissions, prefill starts.  A call that names no prefill instance fails at its
// release, one that names no decode instance or can never fit fails at the end of its prefill; a
// failed call completes at that instant and its workflow is charged the penalty ratio.  Per
// workflow: ratio = completion time * 1000 / SLO; per candidate: their sum, nearest-rank 95th and
// 99th percentiles, the number of late and of failed workflows, the makespan.
//
// The event loop is serial in time, so the parallelism is across candidates (one wavefront each)
// and, inside a step, across calls: the 64 lanes scan the call table for the next instant, apply the
// completions and releases of that instant, and find the best waiting call of an instance by a
// wavefront-wide minimum of (key, index).  Per-call state lives in LDS; the wavefronts of a
// workgroup run their own loops and never meet at a barrier.
struct AgenticParams {
    const uint32_t* arrival;      // [W] microseconds after the earliest arrival
    const unsigned long long* slo;  // [W]
    const uint32_t* wf;           // [K]
    const uint32_t* in_len;       // [K]
    const uint32_t* out_len;      // [K]
    const uint32_t* n_pred;       // [K] number of predecessors
    const uint32_t* succ_first;   // [K + 1] successors of call k: succ[succ_first[k] .. succ_first[k + 1])
    const uint32_t* succ;
    const uint32_t* pa;           // [P] prefill: pa + pb * in_len
    const uint32_t* pb;
    const uint32_t* qc;           // [Q] decode: out_len * (qc + qd * ceil(in_len / 1024))
    const uint32_t* qd;
    const uint32_t* cap;          // [Q]
    unsigned long long penalty;
    uint32_t W, K, P, Q;
    uint32_t wave_bytes;          // LDS per wavefront
};

constexpr uint32_t kAgenticWaves = 4;
constexpr uint32_t kAgenticThreads = kAgenticWaves * kWave;
enum : uint32_t { kBlocked = 0, kWaitPre = 1, kInPre = 2, kWaitDec = 3, kInDec = 4, kDone = 5 };

__device__ __forceinline__ void wave_sync_lds() {
    // LDS writes of any lane of this wavefront are visible to the lanes' later reads; keeps the compiler
    // from carrying LDS values across the point
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
}

// Wavefront-wide reductions on the cross-lane data path of the vector ALU (no trip through LDS, which
// the per-lane shuffles would take): an inclusive scan inside each row of 16 lanes by shifting the row
// right by 1, 2, 4 and 8 lanes (a lane with no source keeps the identity), then the last lane of row 0
// and of row 2 sent to rows 1 and 3, then lane 31 to rows 2 and 3; lane 63 holds the result, which is
// handed to every lane as a uniform value.
#define AP_DPP(identity, v, ctrl, rows) \
    (uint32_t)__builtin_amdgcn_update_dpp((int)(identity), (int)(v), ctrl, rows, 0xF, false)
__device__ __forceinline__ uint32_t wave_all_or(uint32_t v) {
    v |= AP_DPP(0u, v, 0x111, 0xF);                                          // row_shr:1
    v |= AP_DPP(0u, v, 0x112, 0xF);                                          // row_shr:2
    v |= AP_DPP(0u, v, 0x114, 0xF);                                          // row_shr:4
    v |= AP_DPP(0u, v, 0x118, 0xF);                                          // row_shr:8
    v |= AP_DPP(0u, v, 0x142, 0xA);                                          // row_bcast:15 into rows 1 and 3
    v |= AP_DPP(0u, v, 0x143, 0xC);                                          // row_bcast:31 into rows 2 and 3
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}
__device__ __forceinline__ uint32_t wave_all_min(uint32_t v) {
    v = min(v, AP_DPP(kNever, v, 0x111, 0xF));
    v = min(v, AP_DPP(kNever, v, 0x112, 0xF));
    v = min(v, AP_DPP(kNever, v, 0x114, 0xF));
    v = min(v, AP_DPP(kNever, v, 0x118, 0xF));
    v = min(v, AP_DPP(kNever, v, 0x142, 0xA));
    v = min(v, AP_DPP(kNever, v, 0x143, 0xC));
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}
#undef AP_DPP
__device__ __forceinline__ unsigned long long wave_all_or64(unsigned long long v) {
    return ((unsigned long long)wave_all_or((uint32_t)(v >> 32)) << 32) | wave_all_or((uint32_t)v);
}

// Call k has completed: each successor has one predecessor less to wait for.  (Byte counters: the
// decrement goes through the 32-bit word that holds the byte; no borrow can cross into the next
// byte because a counter is decremented exactly as often as it was set.)
__device__ __forceinline__ void agentic_notify(const AgenticParams& p, unsigned char* left, uint32_t k) {
    for (uint32_t i = p.succ_first[k]; i < p.succ_first[k + 1u]; ++i) {
        const uint32_t s = p.succ[i];
        atomicSub(reinterpret_cast<uint32_t*>(left + (s & ~3u)), 1u << ((s & 3u) * 8u));
    }
}

__global__ __launch_bounds__(kAgenticThreads) void k_agentic_eval(AgenticParams p, const uint16_t* __restrict__ pre_inst,
                                                                  const uint16_t* __restrict__ dec_inst,
                                                                  const uint32_t* __restrict__ key,
                                                                  ap_agentic_metrics* __restrict__ out, uint32_t C) {
    extern __shared__ __align__(16) unsigned char lds[];
    const uint32_t lane = threadIdx.x & 63u, wv = wave_index();
    const uint32_t K = p.K, W = p.W;
    unsigned char* mine = lds + wv * p.wave_bytes;
    // per call: event time (end of the running stage, or completion time), key, instance ids, phase
    // (the ratios reuse the key area once the event loop is over; wave_bytes is a multiple of 16)
    uint32_t* ckey = reinterpret_cast<uint32_t*>(mine);          // [max(K, 2 W)]
    unsigned long long* ratio = reinterpret_cast<unsigned long long*>(mine);   // [W]
    uint32_t* tev = ckey + max(K, 2u * W);
    uint32_t* comp = tev + K;                                    // [W] completion time per workflow
    uint32_t* used = comp + W;                                   // [Q] tokens in use
    uint16_t* cpre = reinterpret_cast<uint16_t*>(used + p.Q);
    uint16_t* cdec = cpre + K;
    unsigned char* left = reinterpret_cast<unsigned char*>(cdec + K);   // [K] predecessors still to complete; 4-byte aligned
    unsigned char* phase = left + K;
    unsigned char* busy = phase + K;                             // [P]
    unsigned char* wf_failed = busy + p.P;                       // [W]

    for (uint32_t c = blockIdx.x * kAgenticWaves + wv; c < C; c += gridDim.x * kAgenticWaves) {
        for (uint32_t k = lane; k < K; k += kWave) {
            tev[k] = 0u;
            ckey[k] = key[(size_t)c * K + k];
            cpre[k] = pre_inst[(size_t)c * K + k];
            cdec[k] = dec_inst[(size_t)c * K + k];
            phase[k] = (unsigned char)kBlocked;
            left[k] = (unsigned char)p.n_pred[k];
        }
        for (uint32_t w = lane; w < W; w += kWave) {
            comp[w] = p.arrival[w];                              // a workflow without calls completes on arrival
            wf_failed[w] = 0;
        }
        for (uint32_t q = lane; q < p.Q; q += kWave) used[q] = 0u;
        for (uint32_t i = lane; i < p.P; i += kWave) busy[i] = 0;
        wave_sync_lds();

        // Times are relative to the earliest arrival, so the first instant is 0.  Every step applies the
        // instant's completions, then its releases together with the census of waiting calls and of what
        // happens next, then admissions and starts.  The next instant is the earliest end of a stage in
        // service or arrival of a workflow whose first calls are still to come.
        //
        // Lane l owns the calls l, l + 64, l + 128, ... and keeps three masks over them (bit j: call l + 64 j):
        // not released yet, waiting for an instance, in service.  Only the owner changes a call's phase, so
        // the masks stay in registers, and every scan visits just the calls whose mask bit is set (each lane
        // its own next one per round) instead of the whole table.
        // A fourth mask holds the calls whose workflow has not arrived yet; they are looked at only when
        // the earliest of their arrivals (t_wake) is reached.  That instant is taken as an event whether
        // or not the call is free of predecessors by then; an instant at which nothing can change state
        // changes no result.
        const uint32_t n_mine = lane < K ? (K - lane + kWave - 1u) / kWave : 0u;      // <= 16
        uint32_t m_dormant = (1u << n_mine) - 1u, m_blocked = 0u, m_wait = 0u, m_run = 0u;
        uint32_t t_wake = 0u;                                     // look at them at the first instant
        uint32_t t = 0u;
        for (;;) {
            // ---- 1. completions: decode (frees tokens), prefill (on to the decode queue, or fails) ----
            for (uint32_t m = m_run; __ballot(m != 0u) != 0ull; m &= m - 1u) {
                if (m != 0u) {
                    const uint32_t j = (uint32_t)__ffs((int)m) - 1u, k = lane + kWave * j;
                    if (tev[k] == t) {
                        m_run &= ~(1u << j);
                        if (phase[k] == kInDec) {
                            phase[k] = (unsigned char)kDone;
                            atomicSub(&used[cdec[k]], p.in_len[k] + p.out_len[k]);
                            agentic_notify(p, left, k);
                        } else {                                  // end of its prefill
                            busy[cpre[k]] = 0;
                            const uint32_t q = cdec[k];
                            if (q >= p.Q || p.in_len[k] + p.out_len[k] > p.cap[q]) {
                                phase[k] = (unsigned char)kDone;  // fails here; tev[k] == t is its completion time
                                wf_failed[p.wf[k]] = 1;
                                agentic_notify(p, left, k);
                            } else {
                                phase[k] = (unsigned char)kWaitDec;
                                m_wait |= 1u << j;
                            }
                        }
                    }
                }
            }
            wave_sync_lds();
            // ---- 2. releases, and in the same scan: who is waiting where, what comes next ------------
            // (repeated only when a call failed at its release: it has completed now and may release others)
            if (t_wake <= t) {                                    // workflows of some of my calls have arrived
                t_wake = kNever;
                for (uint32_t m = m_dormant; m != 0u; m &= m - 1u) {
                    const uint32_t j = (uint32_t)__ffs((int)m) - 1u;
                    const uint32_t arrives = p.arrival[p.wf[lane + kWave * j]];
                    if (arrives <= t) {
                        m_dormant &= ~(1u << j);
                        m_blocked |= 1u << j;
                    } else {
                        t_wake = min(t_wake, arrives);
                    }
                }
            }
            unsigned long long dec_waiting, pre_waiting;
            uint32_t t_next;
            for (;;) {
                bool again = false;
                dec_waiting = pre_waiting = 0ull;
                t_next = t_wake;
                for (uint32_t m = m_blocked | m_wait | m_run; __ballot(m != 0u) != 0ull; m &= m - 1u) {
                    if (m != 0u) {
                        const uint32_t j = (uint32_t)__ffs((int)m) - 1u, k = lane + kWave * j;
                        uint32_t ph = phase[k];
                        if (ph == kBlocked) {
                            if (left[k] == 0) {                   // its workflow has arrived: released now
                                m_blocked &= ~(1u << j);
                                if (cpre[k] >= p.P) {
                                    ph = kDone;
                                    tev[k] = t;
                                    wf_failed[p.wf[k]] = 1;
                                    agentic_notify(p, left, k);
                                    again = true;
                                } else {
                                    ph = kWaitPre;
                                    m_wait |= 1u << j;
                                }
                                phase[k] = (unsigned char)ph;
                            }
                        }
                        if (ph == kWaitDec) dec_waiting |= 1ull << cdec[k];
                        if (ph == kWaitPre) pre_waiting |= 1ull << cpre[k];
                        if (ph == kInPre || ph == kInDec) t_next = min(t_next, tev[k]);
                    }
                }
                wave_sync_lds();
                if (__ballot(again) == 0ull) break;
            }
            dec_waiting = wave_all_or64(dec_waiting);
            pre_waiting = wave_all_or64(pre_waiting);
            // ---- 3. decode admissions: the first waiting call of an instance, while it fits --
            while (dec_waiting != 0ull) {
                const uint32_t q = (uint32_t)__ffsll((long long)dec_waiting) - 1u;
                dec_waiting &= dec_waiting - 1ull;
                for (;;) {
                    // smallest (key, index): the smallest key first, then the smallest index among its holders
                    uint32_t best_key = kNever, best_k = kNever;
                    for (uint32_t m = m_wait; __ballot(m != 0u) != 0ull; m &= m - 1u) {
                        if (m != 0u) {
                            const uint32_t k = lane + kWave * ((uint32_t)__ffs((int)m) - 1u);
                            if (phase[k] == kWaitDec && cdec[k] == q && (best_k == kNever || ckey[k] < best_key)) {
                                best_key = ckey[k];               // a lane meets its calls in index order: ties keep the first
                                best_k = k;
                            }
                        }
                    }
                    const uint32_t key_min = wave_all_min(best_key);
                    const uint32_t k = wave_all_min(best_key == key_min ? best_k : kNever);   // the same in every lane
                    if (k == kNever) break;
                    const uint32_t need = p.in_len[k] + p.out_len[k];
                    if (need > p.cap[q] - used[q]) break;              // used <= cap always; the sum could leave 32 bits
                    const uint32_t ends = t + p.out_len[k] * (p.qc[q] + p.qd[q] * ((p.in_len[k] + 1023u) >> 10));
                    t_next = min(t_next, ends);
                    if (lane == (k & 63u)) {                      // its owner
                        used[q] += need;
                        phase[k] = (unsigned char)kInDec;
                        tev[k] = ends;
                        m_wait &= ~(1u << (k >> 6));
                        m_run |= 1u << (k >> 6);
                    }
                    wave_sync_lds();
                }
            }
            // ---- 4. prefill starts on idle instances -------------------------------------------
            while (pre_waiting != 0ull) {
                const uint32_t i = (uint32_t)__ffsll((long long)pre_waiting) - 1u;
                pre_waiting &= pre_waiting - 1ull;
                if (busy[i] != 0) continue;
                uint32_t best_key = kNever, best_k = kNever;
                for (uint32_t m = m_wait; __ballot(m != 0u) != 0ull; m &= m - 1u) {
                    if (m != 0u) {
                        const uint32_t k = lane + kWave * ((uint32_t)__ffs((int)m) - 1u);
                        if (phase[k] == kWaitPre && cpre[k] == i && (best_k == kNever || ckey[k] < best_key)) {
                            best_key = ckey[k];
                            best_k = k;
                        }
                    }
                }
                const uint32_t key_min = wave_all_min(best_key);
                const uint32_t k = wave_all_min(best_key == key_min ? best_k : kNever);   // a call waits there: k is one
                if (k == kNever) continue;
                const uint32_t ends = t + p.pa[i] + p.pb[i] * p.in_len[k];
                t_next = min(t_next, ends);
                if (lane == (k & 63u)) {                          // its owner
                    busy[i] = 1;
                    phase[k] = (unsigned char)kInPre;
                    tev[k] = ends;
                    m_wait &= ~(1u << (k >> 6));
                    m_run |= 1u << (k >> 6);
                }
                wave_sync_lds();
            }
            t = wave_all_min(t_next);
            if (t == kNever) break;
        }

        // ---- workflows -> completion ratios -> metrics --------------------------------------------
        uint32_t last_done = 0u;
        for (uint32_t k = lane; k < K; k += kWave) {
            atomicMax(&comp[p.wf[k]], tev[k]);
            last_done = max(last_done, tev[k]);
        }
        last_done = wave_max_u32(last_done);
        wave_sync_lds();
        unsigned long long sum = 0ull;
        uint32_t n_late = 0u, n_failed = 0u;
        for (uint32_t w = lane; w < W; w += kWave) {
            const unsigned long long took = comp[w] - p.arrival[w];
            const bool failed = wf_failed[w] != 0;
            const unsigned long long r = failed ? p.penalty : took * 1000ull / p.slo[w];
            ratio[w] = r;
            sum += r;
            n_late += (failed || took > p.slo[w]) ? 1u : 0u;
            n_failed += failed ? 1u : 0u;
        }
        sum = wave_sum_u64(sum);
        n_late = wave_sum_u32(n_late);
        n_failed = wave_sum_u32(n_failed);
        wave_sync_lds();
        // nearest rank: the value whose rank among all ratios (ties by workflow index) is the wanted one
        const uint32_t rank95 = (uint32_t)((95ull * W + 99ull) / 100ull) - 1u, rank99 = (uint32_t)((99ull * W + 99ull) / 100ull) - 1u;
        unsigned long long p95 = 0ull, p99 = 0ull;
        for (uint32_t w = lane; w < W; w += kWave) {
            const unsigned long long r = ratio[w];
            uint32_t rank = 0u;
            for (uint32_t v = 0; v < W; ++v) {
                const unsigned long long o = ratio[v];
                rank += (o < r || (o == r && v < w)) ? 1u : 0u;
            }
            if (rank == rank95) p95 = r;
            if (rank == rank99) p99 = r;
        }
        p95 = wave_all_or64(p95);                                // exactly one lane holds each
        p99 = wave_all_or64(p99);
        if (lane == 0u) {
            ap_agentic_metrics m;
            m.sum_ratio_permille = sum;
            m.p95_permille = p95;
            m.p99_permille = p99;
            m.makespan_us = last_done;
            m.n_late = n_late;
            m.n_failed = n_failed;
            out[c] = m;
        }
        wave_sync_lds();
    }
}

}  // namespace

#endif  // AP_AGENTIC_HPP
