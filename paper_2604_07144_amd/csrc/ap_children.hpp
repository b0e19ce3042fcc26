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
constexpr uint32_t kOccupancyThreads = 1024;
constexpr uint32_t kOccupancyWaves = kOccupancyThreads / kWave;
constexpr uint32_t kOccupancyPerThread = 8;       // parent ids per thread and step
constexpr uint32_t kOccupancyStep = kOccupancyThreads * kOccupancyPerThread;
constexpr uint32_t kOccupancyTile = 2u * kOccupancyThreads;                 // requests whose depths are counted together
constexpr uint32_t kOccupancyListCap = kOccupancyStep + kOccupancyTile;

// One workgroup per replica walks the parent row in steps of 8192 ids.  All its threads pick out
// the replica's requests of the step (each thread 8 consecutive ids; counts scanned across the
// workgroup; request indices appended to an LDS list in arrival order).  Whenever the list holds a
// tile of 2048 requests, and once more at the end, the depths of the tile's requests are counted,
// two requests per thread: the depth at a request's arrival is one plus the number of earlier
// requests whose unqueued finish time is later than that arrival.  Earlier requests of the same
// tile are looked at backwards from the request, as far as an arrival plus the tile's longest
// service time still reaches past this arrival (arrivals are in order, so nothing before that can
// still be in service).  Requests of earlier tiles are represented by the 64 latest finish times
// seen so far (`latest`, ascending across the lanes of the first wavefront, kept by dropping the
// earliest and inserting the new one where it belongs): if fewer than 64 earlier requests are
// still in service they are all among those, and 64 or more make the depth exceed every B anyway.
// A depth above 64 is reported as 65.  peak[M] counts the parent's requests that name no replica
// of the table.
__global__ __launch_bounds__(kOccupancyThreads) void k_parent_occupancy(EvalParams p, const uint16_t* __restrict__ parent,
                                                                        uint32_t* __restrict__ peak,
                                                                        uint32_t* __restrict__ room) {
    __shared__ uint32_t list[kOccupancyListCap];  // this replica's requests not yet counted, in arrival order
    __shared__ uint32_t tile_arrival[kOccupancyTile], tile_finish[kOccupancyTile];
    __shared__ uint32_t carry[kWave];             // `latest` as the tile being counted sees it
    __shared__ uint32_t wave_total[kOccupancyWaves];
    __shared__ uint32_t longest;                  // longest service time of the tile
    __shared__ uint32_t wg_deepest;
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wv = wave_index(), m = blockIdx.x;
    const DevReplica rp = p.rep[0];
    uint32_t latest = 0u, deepest = 0u, unknown = 0u, n_list = 0u;
    bool have_carry = false;
    if (tid == 0u) {
        longest = 0u;
        wg_deepest = 0u;
    }

    // Counts the depths of list[0 .. n_tile) and takes them off the list.  Called by all threads with the same
    // arguments; more_follow: requests after this tile may exist, so `latest` has to be brought up to date.
    auto count_tile = [&](uint32_t n_tile, bool more_follow) {
        uint32_t my_arrival[2] = {0u, 0u}, my_longest = 0u;
#pragma unroll
        for (uint32_t q = 0; q < 2u; ++q) {
            const uint32_t i = tid + q * kOccupancyThreads;
            if (i < n_tile) {
                const uint32_t r = list[i];
                uint32_t prefill, tpot;
                request_cost(p.tab_prefill, p.tab_tpot, rp, r, p.prompt[r], prefill, tpot);
                const uint32_t service = prefill + p.outlen[r] * tpot;
                my_arrival[q] = p.arrival[r];
                tile_arrival[i] = my_arrival[q];
                tile_finish[i] = my_arrival[q] + service;
                my_longest = max(my_longest, service);
            }
        }
        my_longest = wave_max_u32(my_longest);
        if (lane == 0u && my_longest != 0u) atomicMax(&longest, my_longest);
        if (wv == 0u) carry[lane] = latest;
        __syncthreads();
        const uint32_t reach = longest;
#pragma unroll
        for (uint32_t q = 0; q < 2u; ++q) {
            const uint32_t i = tid + q * kOccupancyThreads;
            if (i < n_tile) {
                const uint32_t a = my_arrival[q];
                uint32_t depth = 1u;
                if (have_carry)
                    for (uint32_t l = 0; l < kWave; ++l) depth += carry[l] > a ? 1u : 0u;
                for (uint32_t j = i; j > 0u && tile_arrival[j - 1u] + reach > a; --j) depth += tile_finish[j - 1u] > a ? 1u : 0u;
                deepest = max(deepest, min(depth, 65u));
            }
        }
        if (more_follow && wv == 0u) {
            for (uint32_t i0 = 0; i0 < n_tile; i0 += kWave) {
                const uint32_t finish = i0 + lane < n_tile ? tile_finish[i0 + lane] : 0u;
                const uint32_t n_here = min(kWave, n_tile - i0);
                for (uint32_t k = 0; k < n_here; ++k) {
                    const uint32_t f = (uint32_t)__builtin_amdgcn_readlane((int)finish, (int)k);
                    latest = min(wave_shift_down(latest, kNever), max(latest, f));
                }
            }
        }
        __syncthreads();                          // everyone is done with the tile and with list[0 .. n_tile)
        // close the gap: a thread only touches the positions congruent to its own index, front to back
        for (uint32_t d = tid; d + n_tile < n_list; d += kOccupancyThreads) list[d] = list[d + n_tile];
        if (tid == 0u) longest = 0u;
        n_list -= n_tile;
        have_carry = true;
        __syncthreads();
    };

    // my 8 ids of a step: one 16-byte load where the row has them all (the parent buffer is 16-byte aligned
    // and a thread's run starts at a multiple of 8 ids), one by one at the ragged end
    auto fetch = [&](uint4& into, uint32_t r0) {
        const uint32_t at = r0 + tid * kOccupancyPerThread;
        if (at + kOccupancyPerThread <= p.R) {
            into = *reinterpret_cast<const uint4*>(parent + at);
        } else {
            uint32_t w[4];
#pragma unroll
            for (uint32_t k = 0; k < 4u; ++k) {
                const uint32_t lo = at + 2u * k < p.R ? (uint32_t)parent[at + 2u * k] : 0xFFFFu;
                const uint32_t hi = at + 2u * k + 1u < p.R ? (uint32_t)parent[at + 2u * k + 1u] : 0xFFFFu;
                w[k] = lo | (hi << 16);
            }
            into = make_uint4(w[0], w[1], w[2], w[3]);
        }
    };
    uint4 ids_next;
    fetch(ids_next, 0u);
    __syncthreads();                              // longest and wg_deepest are set
    for (uint32_t r0 = 0; r0 < p.R; r0 += kOccupancyStep) {
        // as a bit mask: which of my 8 ids name this replica (absent ones read as 0xFFFF and are skipped below)
        const uint32_t mine = r0 + tid * kOccupancyPerThread;
        const uint32_t w[4] = {ids_next.x, ids_next.y, ids_next.z, ids_next.w};
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
        uint32_t at = n_list + upto - n_mine, n_step = 0u;
#pragma unroll
        for (uint32_t j = 0; j < kOccupancyWaves; ++j) {
            at += j < wv ? wave_total[j] : 0u;
            n_step += wave_total[j];
        }
        for (uint32_t h = hits; h != 0u; h &= h - 1u) list[at++] = mine + (uint32_t)__ffs((int)h) - 1u;
        n_list += n_step;                         // below kOccupancyListCap: less than a tile was left over
        __syncthreads();                          // the list is written; wave_total may be rewritten
        const bool last_step = r0 + kOccupancyStep >= p.R;
        while (n_list >= kOccupancyTile) count_tile(kOccupancyTile, !(last_step && n_list == kOccupancyTile));
        if (last_step && n_list > 0u) count_tile(n_list, false);
    }
    deepest = wave_max_u32(deepest);
    if (lane == 0u) atomicMax(&wg_deepest, deepest);
    __syncthreads();
    if (tid == 0u) {
        const uint32_t d = wg_deepest;
        peak[m] = d;
        room[m] = d <= p.B ? p.B - d : 0u;
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
