// Exact replay, fused: k_eval_candidates.
#ifndef AP_REPLAY_HPP
#define AP_REPLAY_HPP

#include "ap_common.hpp"

namespace {

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
// kTabled: prefill time and time per token come from the caller's tables (one pair of loads per
// request in the replay step) instead of the linear stand-in; prompt lengths are then not staged.
template <bool kHist16, bool kLen16, bool kTabled>
__global__ __launch_bounds__(kThreads) void k_eval_candidates(EvalParams p, const uint16_t* __restrict__ assign,
                                                              ap_metrics* out, uint32_t C, uint32_t only_pending,
                                                              PendingWord flags) {
    if (only_pending && pending_none(flags)) return;  // the kernels before this one have left no mark
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
        if (tid == 0u) atomicAdd(p.replayed, 1u);

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
                kprompt[g] = kTabled ? 0u : p.prompt[r0 + idx];
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
                    if (!kTabled) c_prompt[idx] = (len_t)kprompt[g];
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
                    const uint32_t arr = c_arr[li], ol = c_out[li];                         // widened to 32 bits
                    const uint32_t ready = max(arr, rp.t_on);
                    uint32_t prefill, tpot;
                    request_cost<kTabled>(p.tab_prefill, p.tab_tpot, rp, r0 + li, kTabled ? 0u : (uint32_t)c_prompt[li],
                                          prefill, tpot);
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
                                // the same when every request of the run is ready before the first slot frees (a
                                // backlog): the earliest slot time only grows, so each starts when that slot frees
                                auto step_backlog = [&](uint32_t j) {
                                    const uint32_t u = (uint32_t)__builtin_amdgcn_readfirstlane((int)S);
                                    const uint32_t fj = u + (uint32_t)__builtin_amdgcn_readlane((int)svc, (int)j);
                                    S = min(wave_shift_down(S, kNever), max(S, fj));
                                    pushed = wave_shift_up(pushed, u);
                                };
                                uint32_t j = n_first;
                                const bool backlog = (uint32_t)__builtin_amdgcn_readlane((int)ready, (int)(n_run - 1u)) <=
                                                     (uint32_t)__builtin_amdgcn_readfirstlane((int)S);   // ready times do not decrease
                                if (backlog) {
                                    for (; j + 2u <= n_run; j += 2u) {
                                        step_backlog(j);
                                        step_backlog(j + 1u);
                                    }
                                    if (j < n_run) step_backlog(j);
                                } else {
                                    for (; j + 2u <= n_run; j += 2u) {
                                        step(j);
                                        step(j + 1u);
                                    }
                                    if (j < n_run) step(j);
                                }
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

}  // namespace

#endif  // AP_REPLAY_HPP
