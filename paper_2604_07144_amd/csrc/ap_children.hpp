// Sparse candidates: parent occupancy and the per-child shortcut / row writer.
#ifndef AP_CHILDREN_HPP
#define AP_CHILDREN_HPP

#include "ap_common.hpp"

namespace {

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
                    uint32_t prefill, tpot;
                    request_cost(p.tab_prefill, p.tab_tpot, rp, r, p.prompt[r], prefill, tpot);
                    arrival = p.arrival[r];
                    finish = arrival + prefill + p.outlen[r] * tpot;
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
                                                                    ap_metrics* __restrict__ out, uint32_t C,
                                                                    PendingWord flags) {
    extern __shared__ __align__(16) unsigned char lds[];
    pending_clear_next(flags);
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
            if (dense && lane == 0u) pending_raise(flags);
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

#endif  // AP_CHILDREN_HPP
