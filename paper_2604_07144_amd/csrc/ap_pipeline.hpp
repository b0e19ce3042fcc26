// Exact replay as three kernels for large replica tables: group -> replay -> reduce.
#ifndef AP_PIPELINE_HPP
#define AP_PIPELINE_HPP

#include "ap_common.hpp"

namespace {

// ----------------------------------------------------------------------------------
// exact replay as three kernels: group -> replay -> reduce
// ----------------------------------------------------------------------------------
// The candidates of a batch are scored by three kernels that hand their intermediates over
// in a device scratch area sized once by ap_costmodel_set (about 1 GiB, cut into whole
// candidates: enough of them per launch to fill the device; every intermediate is written once
// and read once, so the area is not meant to stay in cache):
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
    uint32_t* replayed;                // device counter: candidates that went through the exact replay kernels
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
        if (tid == 0u) atomicAdd(p.replayed, 1u);
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
    const uint32_t* tab_prefill;       // cost tables, or null (see EvalParams)
    const uint32_t* tab_tpot;
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
                        uint32_t prefill, tpot;
                        request_cost(p.tab_prefill, p.tab_tpot, rp, r, rq.y, prefill, tpot);
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

}  // namespace

#endif  // AP_PIPELINE_HPP
