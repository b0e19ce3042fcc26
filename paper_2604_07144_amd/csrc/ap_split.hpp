// Exact evaluation for replicas that differ or come and go: the trace of every replica is cut in two.
#ifndef AP_SPLIT_HPP
#define AP_SPLIT_HPP

#include <type_traits>

#include "ap_common.hpp"
#include "ap_screen.hpp"

namespace {

// ----------------------------------------------------------------------------------
// split evaluation: a listed part that is replayed, a streamed part that provably never waits
// ----------------------------------------------------------------------------------
// Replica m serves during [t_on, t_off) (the snapshot holds cluster availability, Section 4; Section 8.2
// "Elastic Cluster Dynamics").  Requests are in arrival order, so for every replica three index ranges are
// fixed by the trace alone, whatever the candidate:
//   r >= i_off[m]             arrives when the replica is gone: rejected on arrival;
//   r <  i_list[m]            the LISTED part: everything that arrives before the replica is up (its backlog)
//                             and while that backlog drains.  These requests are grouped by replica and
//                             replayed exactly through the B-slot queue (k_replay_lists);
//   i_list[m] <= r < i_off[m] the STREAMED part: scored where the assignment row is read, as requests that
//                             start on arrival (ttft = prefill), without a queue.
// Why the streamed part may skip the queue.  Let D(r) be the number of requests r' <= r of the whole trace,
// on any replica, whose service interval [arrival, arrival + longest service over the replica kinds) holds
// arrival(r): no candidate can have more requests that started on arrival in service on one replica at that
// moment.  Let busy(c, m) be the number of slots of replica m that the listed part of candidate c leaves taken
// beyond t_split[m] = arrival(i_list[m]).  If busy(c, m) + max over r >= i_list[m] of D(r) <= B, then by
// induction in arrival order every streamed request of (c, m) finds a free slot when it arrives: the requests
// of m in service at that moment are listed ones still running (at most busy) and earlier streamed ones, which
// started on arrival by the induction hypothesis and are therefore counted by D(r) - 1.  The host picks
// i_list[m] so that the bound leaves room (ap_costmodel_set); k_replay_lists counts busy(c, m) at the end of
// every list and hands the candidate to the general replay if the room is not there.  A trace too dense for
// any room (D above B) simply has every request listed.
//
// Per candidate the record is put together from three parts that add up (sums, counts) or combine by max
// (latest finish): the streamed part (k_split_candidates), the listed part (k_replay_lists, one atomic update per
// queue) and the rejected requests at the penalty latency (k_merge_candidates).
//
// The p99 fields need the histograms only when fewer than R - k99 + 1 requests are rejected.  Otherwise the
// k99-th smallest value of each metric is the penalty latency itself (rejected requests are charged it,
// Appendix "Serving Simulator", Memory Feasibility), provided every served latency falls in a lower bin, which
// the host checks against its bound on all finish times.  Such a candidate is called settled-by-penalty below
// and carries kFlagLazy; the others keep histograms: the streamed requests are counted in LDS while the row is
// read (and parked in device memory), the list replay leaves the bins of every listed request next to its list
// entry, and k_merge_candidates adds the two up.
constexpr uint32_t kSplitWaves = 4;
constexpr uint32_t kSplitThreads = kSplitWaves * kWave;
constexpr uint32_t kTile = 1024;                  // requests per tile: a list position fits 10 bits
constexpr uint32_t kFlagNeedHist = 1u;            // streamed without histograms, but they are needed: stream again
constexpr uint32_t kFlagFallback = 2u;            // the listed part left too many slots taken: general replay
constexpr uint32_t kFlagLazy = 4u;                // the p99 values are the penalty latency
constexpr uint32_t kFlagNoStreamHist = 8u;        // histograms needed, and no request of the candidate was streamed
constexpr uint32_t kBinServed = 0x80000000u;      // bins word of a listed request: ttft bin | e2e bin << 12 | this if served

// Per replica, for the streaming kernel, as three arrays (copied to LDS; an entry per replica and one more, index
// M, for unknown replica ids: everything rejected).  Lanes look entries up by replica id, so consecutive ids must
// fall into different LDS banks: one 32-bit word per replica holds both ranges when R is below 65536 (else one
// word each), and the cost coefficients are stored once per kind of replica, which another word names.
struct SplitTables {
    const uint32_t* range;                        // [M + 1] i_list | i_off << 16; wide: i_list
    const uint32_t* range_off;                    // wide only: [M + 1] i_off
    const uint32_t* kind;                         // [M + 1] index into coef; tabulated cost model: the replica's type
                                                  //   (either way below 1024: it rides in the upper bits of a tile word)
    const uint4* coef;                            // [n_kinds] a, b, c, d
    uint32_t n_kinds;
};

struct SplitQueue {                               // per replica, for the list replay, 48 bytes
    uint32_t a, b, c, d, t_on, t_off;
    uint32_t i_list;
    uint32_t t_split;                             // arrival of request i_list; kNever: nothing is streamed
    uint32_t allow_busy;                          // slots that may still be taken beyond t_split
    uint32_t pad0, pad1, pad2;
};

struct SplitPartial {                             // per candidate of a batch, 64 bytes
    unsigned long long s_e2e, s_ttft, s_tpot;     // served requests only
    uint32_t last_fin, n_ok, n_rej, flags;
    uint32_t pad[6];
};

struct SplitParams {
    const uint2* req8;                            // [R] {arrival, prompt | out << 16}
    SplitTables tab;
    const SplitQueue* queue;                      // [M]
    const uint32_t* order;                        // [n_queues] replicas with a listed part, longest first
    uint32_t* desc;                               // [batch][n_list_tiles][M + 1] count << 16 | first list position of
                                                  //   the replica's run; entry M: list positions the tile uses in all
    uint16_t* lists;                              // [batch][n_list_tiles][tile_cap] tile-local request indices by replica
    SplitPartial* part;                           // [batch]
    uint32_t* hist;                               // [batch][hist_words] the streamed requests' histograms
    uint2* bins;                                  // [batch][n_list_tiles][tile_cap] bins of every listed request:
                                                  //   x = ttft bin | e2e bin << 12 | kBinServed, y = tpot bin
    const uint2* tab_pair;                        // tabulated cost model: [T][R] {prefill time, time per token}; the kind
                                                  //   word of a replica then holds its type, SplitQueue::a type * R
    uint32_t hist_words;                          // 3 * kBins / 2 (16-bit counts, R < 65536) or 3 * kBins
    uint32_t wide;                                // R >= 65536: two range words per replica
    uint32_t any_streamed;                        // some replica has a streamed part
    uint32_t R, M, B, key_bits;
    uint32_t n_tiles, n_list_tiles, tile_cap, n_queues;
    uint32_t slo_ttft, slo_tpot;
    uint32_t lazy_from;                           // rejected requests from which the p99 values are the penalty; kNever: never
    uint32_t all_within;                          // no request's prefill or time per token can exceed the objectives
    // byte offsets into the streaming kernel's dynamic LDS
    uint32_t off_range, off_range_off, off_kind, off_coef, off_acc, off_wave, wave_bytes, w_pos, w_queue, w_list, w_same, w_tile,
        off_hist;
};

// The two cost tables of a tabulated model side by side, so that a request's prefill time and time per token come
// with one 8-byte load.
__global__ __launch_bounds__(kThreads) void k_pair_tables(const uint32_t* __restrict__ prefill, const uint32_t* __restrict__ tpot,
                                                          uint2* __restrict__ pair, size_t n) {
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += (size_t)gridDim.x * kThreads)
        pair[i] = make_uint2(prefill[i], tpot[i]);
}

// Streaming kernel.  One workgroup per candidate at a time; its wavefronts take the tiles of the row in turn
// and share nothing but the accumulators (and the histograms), so there is no barrier inside a candidate.
// Per tile a wavefront classifies its 1024 requests, accumulates the streamed ones, counts the listed ones per
// replica, queues them in arrival order, ranks them (one ballot per bit of the replica id among 64 queued
// requests at a time) into per-replica runs that start on multiples of 8 list positions, and writes the runs
// and their descriptors out.
// kHistMode: 0 keeps no histograms of the streamed requests (enough when the candidate is settled by penalty, or
// when nothing is streamed at all), 1 keeps them with 16-bit counts (R < 65536), 2 with 32-bit counts.
// only_flagged: look only at candidates that an earlier launch marked kFlagNeedHist.
// kNarrow: at most 64 replicas, so a queued request (tile index and replica) fits 16 bits, which halves the queue.
// kTabled: prefill time and time per token are read from the tables (one 8-byte load per request, issued with the
// table look-ups of the quarter tile) instead of being evaluated from a kind's coefficients.
template <uint32_t kHistMode, bool kNarrow, bool kTabled>
__global__ __launch_bounds__(kSplitThreads, 5) void k_split_candidates(SplitParams p, const uint16_t* __restrict__ assign,
                                                                    uint32_t c0, uint32_t n_cand, uint32_t only_flagged,
                                                                    PendingWord flags) {
    extern __shared__ __align__(16) unsigned char lds[];
    pending_clear_next(flags);
    constexpr bool kHist = kHistMode != 0u, kHist16 = kHistMode == 1u;
    uint32_t* hist = reinterpret_cast<uint32_t*>(lds + p.off_hist);          // kHist only
    uint32_t* range_of = reinterpret_cast<uint32_t*>(lds + p.off_range);
    uint32_t* range_off_of = reinterpret_cast<uint32_t*>(lds + p.off_range_off);   // wide only
    uint32_t* kind_of = reinterpret_cast<uint32_t*>(lds + p.off_kind);
    uint4* coef_of = reinterpret_cast<uint4*>(lds + p.off_coef);
    unsigned long long* acc64 = reinterpret_cast<unsigned long long*>(lds + p.off_acc);
    uint32_t* acc32 = reinterpret_cast<uint32_t*>(lds + p.off_acc + 24);    // latest finish, within objectives, rejected
    const uint32_t tid = threadIdx.x, lane = tid & 63u, w = wave_index();
    unsigned char* mine = lds + p.off_wave + w * p.wave_bytes;
    uint32_t* cnt = reinterpret_cast<uint32_t*>(mine);                       // [M] listed requests of the tile per replica
    uint32_t* pos = reinterpret_cast<uint32_t*>(mine + p.w_pos);             // [M] next free position of the replica's run
    using queued_t = typename std::conditional<kNarrow, uint16_t, uint32_t>::type;
    constexpr uint32_t kIdShift = kNarrow ? 10u : 16u;
    queued_t* queue = reinterpret_cast<queued_t*>(mine + p.w_queue);         // [kTile] tile index | replica << kIdShift, arrival order
    uint16_t* list = reinterpret_cast<uint16_t*>(mine + p.w_list);           // [tile_cap]
    unsigned long long* same = reinterpret_cast<unsigned long long*>(mine + p.w_same);   // [M] lanes naming the replica
    uint32_t* tile_of = reinterpret_cast<uint32_t*>(mine + p.w_tile);        // [M + 1] the replica's ranges within the tile in hand
    const uint32_t R = p.R, M = p.M;

    if (only_flagged) {                                                             // usually nothing is: leave at once
        bool any = false;
        for (uint32_t cb = blockIdx.x; cb < n_cand; cb += gridDim.x) any = any || (p.part[cb].flags & kFlagNeedHist) != 0u;
        if (!any) return;                                                           // the same words for every thread
    }
    for (uint32_t i = tid; i <= M; i += kSplitThreads) {
        range_of[i] = p.tab.range[i];
        if (p.wide != 0u) range_off_of[i] = p.tab.range_off[i];
        kind_of[i] = p.tab.kind[i];
    }
    for (uint32_t i = tid; i < p.tab.n_kinds; i += kSplitThreads) coef_of[i] = p.tab.coef[i];
    for (uint32_t m = lane; m < M; m += kWave) {
        cnt[m] = 0u;
        same[m] = 0ull;
    }

    for (uint32_t cb = blockIdx.x; cb < n_cand; cb += gridDim.x) {
        if (only_flagged && (p.part[cb].flags & kFlagNeedHist) == 0u) continue;     // the same word for every thread
        __syncthreads();                                                            // the last candidate's totals were read
        if (kHist)
            for (uint32_t i = tid; i < p.hist_words; i += kSplitThreads) hist[i] = 0u;
        if (tid < 10u) reinterpret_cast<uint32_t*>(acc64)[tid] = 0u;
        __syncthreads();
        const uint16_t* row = assign + (size_t)(c0 + cb) * R;
        const bool row_aligned = (reinterpret_cast<uintptr_t>(row) & 3u) == 0u;      // pairs of ids as one 4-byte load
        unsigned long long s_e2e = 0, s_ttft = 0, s_tpot = 0;
        uint32_t last_fin = 0, n_ok = 0, n_rej = 0;

        // A wavefront's tiles.  A lane holds two consecutive requests of every 128 (one 4-byte load of two replica
        // ids, one 16-byte load of two request records).  The ids of the next tile are requested before the current
        // one is worked on and the records of a quarter tile before that quarter; the table look-ups of a quarter are issued
        // together, so that no request waits for memory or for the LDS by itself.
        constexpr uint32_t kPairs = kTile / (2u * kWave), kParts = 4u, kHalf = kPairs / kParts;   // pairs per lane and tile; per part
        uint32_t key[kPairs], key_next[kPairs];
        auto fetch_keys = [&](uint32_t (&into)[kPairs], uint32_t j) {
            const uint32_t r0 = j * kTile;
            if (r0 + kTile <= R && row_aligned) {                                   // a whole tile: no guards
#pragma unroll
                for (uint32_t g = 0; g < kPairs; ++g)
                    into[g] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(row + r0 + g * 2u * kWave + 2u * lane));
            } else {
                const uint32_t n = r0 < R ? min(kTile, R - r0) : 0u;
#pragma unroll
                for (uint32_t g = 0; g < kPairs; ++g) {
                    const uint32_t rl = g * 2u * kWave + 2u * lane;
                    const uint32_t lo = rl < n ? (uint32_t)__builtin_nontemporal_load(row + r0 + rl) : 0u;
                    const uint32_t hi = rl + 1u < n ? (uint32_t)__builtin_nontemporal_load(row + r0 + rl + 1u) : 0u;
                    into[g] = lo | (hi << 16);
                }
            }
        };
        // one tile; kWhole: all of its 1024 requests exist
        auto work_tile = [&](auto whole_tag, uint32_t j) {
            constexpr bool kWhole = decltype(whole_tag)::value;
            const uint32_t r0 = j * kTile, n = min(kTile, R - r0);
            const bool grouping = j < p.n_list_tiles;                               // beyond: nothing can be listed
            // The replica ranges cut down to this tile, one word per replica: listed below position `lo` of the tile,
            // gone from position `hi` on (both 0 .. 1024, 11 bits each), and the replica's kind
            // above them (or its type, when the costs come from tables), so that a request needs one look-up.
            // (The wavefront's own LDS accesses execute in order.)
            for (uint32_t m = lane; m <= M; m += kWave) {
                const uint32_t word = range_of[m];
                const uint32_t i_list = p.wide != 0u ? word : (word & 0xFFFFu);
                const uint32_t i_off = p.wide != 0u ? range_off_of[m] : (word >> 16);
                const uint32_t lo = min(max(i_list, r0) - r0, kTile), hi = min(max(i_off, r0) - r0, kTile);
                tile_of[m] = lo | (hi << 11) | (kind_of[m] << 22);
            }
            uint32_t q_n = 0;                                                       // queued so far (the same in every lane)
            uint32_t t_e2e = 0, t_ttft = 0, t_tpot = 0;                             // the tile's sums: 16 values below 2^28 each
#pragma unroll
            for (uint32_t h = 0; h < kParts; ++h) {
                uint4 record[kHalf];
                uint32_t id[2u * kHalf], from[2u * kHalf], upto[2u * kHalf], kind[2u * kHalf];   // listed below `from`, gone from `upto`
                uint32_t cost_prefill[kTabled ? 2u * kHalf : 1u], cost_tpot[kTabled ? 2u * kHalf : 1u];
#pragma unroll
                for (uint32_t g = 0; g < kHalf; ++g) {
                    const uint32_t rl = (h * kHalf + g) * 2u * kWave + 2u * lane;
                    record[g] = (kWhole || rl < n) ? *reinterpret_cast<const uint4*>(p.req8 + r0 + rl) : make_uint4(0u, 0u, 0u, 0u);
                    id[2u * g] = min(key[h * kHalf + g] & 0xFFFFu, M);
                    id[2u * g + 1u] = min(key[h * kHalf + g] >> 16, M);
                }
#pragma unroll
                for (uint32_t i = 0; i < 2u * kHalf; ++i) {
                    const uint32_t word = tile_of[id[i]];
                    from[i] = word & 0x7FFu;
                    upto[i] = (word >> 11) & 0x7FFu;
                    kind[i] = kTabled ? (word >> 22) * R : word >> 22;       // tabulated: the type's first table entry
                }
                if (kTabled) {
#pragma unroll
                    for (uint32_t i = 0; i < 2u * kHalf; ++i) {                     // whether streamed or not: the entry exists
                        const uint32_t r = min(r0 + (h * kHalf + (i >> 1)) * 2u * kWave + 2u * lane + (i & 1u), R - 1u);
                        const uint2 cost = p.tab_pair[kind[i] + r];
                        cost_prefill[i] = cost.x;
                        cost_tpot[i] = cost.y;
                    }
                }
#pragma unroll
                for (uint32_t g = 0; g < kHalf; ++g) {
                    bool listed[2];
#pragma unroll
                    for (uint32_t e = 0; e < 2u; ++e) {
                        const uint32_t i = 2u * g + e;
                        const uint32_t rl = (h * kHalf + g) * 2u * kWave + 2u * lane + e;
                        const bool in = kWhole || rl < n;
                        listed[e] = in && rl < from[i];                             // lo <= hi
                        const bool rejected = in && rl >= upto[i];
                        const bool streamed = in && !listed[e] && !rejected;
                        n_rej += (uint32_t)__popcll(__ballot(rejected));
                        if (p.all_within != 0u) n_ok += (uint32_t)__popcll(__ballot(streamed));   // a wavefront total then
                        if (streamed) {
                            // starts on arrival: ttft = prefill
                            const uint32_t arrival = e ? record[g].z : record[g].x, lens = e ? record[g].w : record[g].y;
                            const uint32_t prompt = lens & 0xFFFFu, out = lens >> 16;
                            uint32_t prefill, tpot;
                            if (kTabled) {
                                prefill = cost_prefill[i];
                                tpot = cost_tpot[i];
                            } else {
                                const uint4 co = coef_of[kind[i]];
                                prefill = co.x + __umul24(co.y, prompt);            // the host keeps all factors below 2^24
                                tpot = co.z + __umul24(co.w, (prompt + 1023u) >> 10);
                            }
                            const uint32_t e2e = prefill + __umul24(out, tpot);
                            t_ttft += prefill;
                            t_e2e += e2e;
                            t_tpot += tpot;
                            last_fin = max(last_fin, arrival + e2e);
                            if (p.all_within == 0u) n_ok += (prefill <= p.slo_ttft && tpot <= p.slo_tpot) ? 1u : 0u;
                            if (kHist) {
                                hist_add<kHist16>(hist, 0u, hist_bin_u32(prefill), 1u);
                                hist_add<kHist16>(hist, 1u, hist_bin_u32(tpot), 1u);
                                hist_add<kHist16>(hist, 2u, hist_bin_u32(e2e), 1u);
                            }
                        }
                    }
                    // queue the listed ones in arrival order: lanes in order, a lane's first request before its second
                    const unsigned long long lm0 = __ballot(listed[0]), lm1 = __ballot(listed[1]);
                    const uint32_t before = __builtin_amdgcn_mbcnt_hi((uint32_t)(lm0 >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)lm0, 0u)) +
                                            __builtin_amdgcn_mbcnt_hi((uint32_t)(lm1 >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)lm1, 0u));
                    const uint32_t rl = (h * kHalf + g) * 2u * kWave + 2u * lane;
                    if (listed[0]) {
                        atomicAdd(&cnt[id[2u * g]], 1u);
                        queue[q_n + before] = (queued_t)(rl | (id[2u * g] << kIdShift));
                    }
                    if (listed[1]) {
                        atomicAdd(&cnt[id[2u * g + 1u]], 1u);
                        queue[q_n + before + (listed[0] ? 1u : 0u)] = (queued_t)((rl + 1u) | (id[2u * g + 1u] << kIdShift));
                    }
                    q_n += (uint32_t)__popcll(lm0) + (uint32_t)__popcll(lm1);
                }
            }
            s_ttft += t_ttft;
            s_e2e += t_e2e;
            s_tpot += t_tpot;
            if (!grouping) return;                                                  // q_n is 0 there
            // runs: every replica's listed requests of the tile, starting on a multiple of 8 positions
            const size_t tile_at = (size_t)cb * p.n_list_tiles + j;
            uint32_t total = 0;
            for (uint32_t base = 0; base < M; base += kWave) {
                const uint32_t m = base + lane;
                const uint32_t c = m < M ? cnt[m] : 0u;
                const uint32_t room = (c + 7u) & ~7u;
                const uint32_t upto = wave_inclusive_scan(room, lane);
                if (m < M) {
                    pos[m] = total + upto - room;
                    cnt[m] = 0u;                                                    // for the wavefront's next tile
                    p.desc[tile_at * (M + 1u) + m] = (c << 16) | (total + upto - room);
                }
                total += (uint32_t)__builtin_amdgcn_readlane((int)upto, 63);
            }
            if (lane == 0u) p.desc[tile_at * (M + 1u) + M] = total;
            // Rank among the queued requests of one replica, 64 queued requests at a time: every lane sets its bit
            // in its replica's word and reads the word back (the LDS executes a wavefront's instructions in order),
            // which tells it how many lanes before it name the same replica; the last of them moves the run's
            // position on and clears the word.
            for (uint32_t d0 = 0; d0 < q_n; d0 += kWave) {
                if (d0 + lane < q_n) {
                    const uint32_t pair = queue[d0 + lane];
                    const uint32_t k = pair >> kIdShift;
                    atomicOr(&same[k], 1ull << lane);
                    const unsigned long long peers = same[k];
                    const uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(peers >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)peers, 0u));
                    const uint32_t n_peers = (uint32_t)__popcll(peers);
                    const uint32_t at = pos[k];
                    list[at + rank] = (uint16_t)(pair & (kTile - 1u));
                    if (rank + 1u == n_peers) {
                        pos[k] = at + n_peers;
                        same[k] = 0ull;
                    }
                }
            }
            // 16 bytes (8 positions) at a time; the padding of a run holds whatever the LDS held
            uint4* dst = reinterpret_cast<uint4*>(p.lists + tile_at * p.tile_cap);
            for (uint32_t v = lane; v < total / 8u; v += kWave) dst[v] = reinterpret_cast<const uint4*>(list)[v];
        };
        fetch_keys(key_next, w);
        for (uint32_t j = w; j < p.n_tiles; j += kSplitWaves) {
#pragma unroll
            for (uint32_t g = 0; g < kPairs; ++g) key[g] = key_next[g];
            fetch_keys(key_next, j + kSplitWaves);
            if ((j + 1u) * kTile <= R) work_tile(std::true_type{}, j);
            else work_tile(std::false_type{}, j);
        }

        // the workgroup's totals
        s_e2e = wave_sum_u64(s_e2e);
        s_ttft = wave_sum_u64(s_ttft);
        s_tpot = wave_sum_u64(s_tpot);
        last_fin = wave_max_u32(last_fin);
        if (p.all_within == 0u) n_ok = wave_sum_u32(n_ok);                          // else counted per wavefront already
        if (lane == 0u) {
            atomicAdd(&acc64[0], s_e2e);
            atomicAdd(&acc64[1], s_ttft);
            atomicAdd(&acc64[2], s_tpot);
            atomicMax(&acc32[0], last_fin);
            atomicAdd(&acc32[1], n_ok);
            atomicAdd(&acc32[2], n_rej);                                            // already a wavefront total
        }
        __syncthreads();
        const uint32_t rejected = acc32[2];
        const bool lazy = rejected >= p.lazy_from;
        if (tid == 0u) {
            SplitPartial sp{};
            sp.s_e2e = acc64[0];
            sp.s_ttft = acc64[1];
            sp.s_tpot = acc64[2];
            sp.last_fin = acc32[0];
            sp.n_ok = acc32[1];
            sp.n_rej = rejected;
            sp.flags = lazy ? kFlagLazy : (kHist ? 0u : (p.any_streamed != 0u ? kFlagNeedHist : kFlagNoStreamHist));
            p.part[cb] = sp;
        }
        if (kHist && !lazy) {
            uint32_t* dst = p.hist + (size_t)cb * p.hist_words;
            for (uint32_t i = tid; i < p.hist_words; i += kSplitThreads) dst[i] = hist[i];
        }
    }
}

// The median of three: with a <= c it is min(c, max(a, b)), in one instruction.
__device__ __forceinline__ uint32_t median3(uint32_t a, uint32_t b, uint32_t c) {
    uint32_t r;
    asm("v_med3_u32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// List replay.  One lane per (candidate, replica) queue: the 64 lanes of a wavefront replay the listed part of
// replica m under 64 candidates of the batch, and the kListWaves wavefronts of a workgroup take neighbouring
// candidates of the same replica.  All lanes share the replica, hence its cost coefficients and window (scalar
// registers) and - roughly - the pace at which they move through the trace, so the request records of
// kReplayTiles tiles are staged in LDS once per workgroup and read by every lane; inside such a stage the
// wavefronts run free (no barrier), and within a wavefront the lanes meet again at every tile, where the lane
// with the most requests of the tile sets the pace.  Staging several tiles at a time for several wavefronts is
// what keeps the share of idle lane-steps down: the counts of a stage differ less, relative to their mean, than
// those of a single tile.
// A lane keeps its B slot-free times sorted in registers (s[0] the earliest); a request starts at
// max(ready, s[0]), and its finish time f replaces s[0] by one median per register:
// s'[i] = med3(s[i], f, s[i+1]), i.e. min(s[i+1], max(s[i], f)).  A lane without a request in a step (or whose
// request is rejected) inserts 0, which leaves the registers as they are.
// Starts do not decrease along a queue, so once a start reaches t_off every later request is rejected too.
// kSlots: B rounded up to a power of two; registers beyond B hold kNever and stay there.
// kBinsOut: the variant that leaves the histogram bins of its requests for the merge.  which: 0 every
// candidate, 1 only those settled by penalty (the lean variant's share), 2 only the others; a workgroup
// without a lane to work on ends at once.
constexpr uint32_t kListWaves = 4;
constexpr uint32_t kReplayListThreads = kListWaves * kWave;
constexpr uint32_t kReplayTiles = 2;              // tiles staged at a time: 16 KiB of request records per workgroup

// kTabled: a staged record carries the request's prefill time and time per token on this replica's type, read
// from the tables while staging, instead of its lengths.
template <uint32_t kSlots, bool kBinsOut, bool kTabled>
__global__ __launch_bounds__(kReplayListThreads) void k_replay_lists(SplitParams p, uint32_t n_cand, uint32_t which) {
    using staged_t = typename std::conditional<kTabled, uint4, uint2>::type;         // {arrival, out, prefill, tpot} or {arrival, lengths}
    __shared__ staged_t recs[kReplayTiles * kTile];
    const uint32_t tid = threadIdx.x;
    const uint32_t n_blocks = (n_cand + kReplayListThreads - 1u) / kReplayListThreads;
    const uint32_t m = p.order[blockIdx.x / n_blocks];
    const uint32_t cb = (blockIdx.x % n_blocks) * kReplayListThreads + tid;
    bool live = cb < n_cand;
    const bool lazy = live && (p.part[cb].flags & kFlagLazy) != 0u;
    if (which == 1u) live = lazy;
    if (which == 2u) live = live && !lazy;
    if (__syncthreads_or(live ? 1 : 0) == 0) return;
    const bool with_hist = kBinsOut && live && !lazy;                               // leave the bins of every request
    SplitQueue q = p.queue[m];
    q.a = (uint32_t)__builtin_amdgcn_readfirstlane((int)q.a);
    q.b = (uint32_t)__builtin_amdgcn_readfirstlane((int)q.b);
    q.c = (uint32_t)__builtin_amdgcn_readfirstlane((int)q.c);
    q.d = (uint32_t)__builtin_amdgcn_readfirstlane((int)q.d);
    q.t_on = (uint32_t)__builtin_amdgcn_readfirstlane((int)q.t_on);
    q.t_off = (uint32_t)__builtin_amdgcn_readfirstlane((int)q.t_off);
    q.i_list = (uint32_t)__builtin_amdgcn_readfirstlane((int)q.i_list);

    uint32_t s[kSlots];
#pragma unroll
    for (uint32_t i = 0; i < kSlots; ++i) s[i] = i < p.B ? 0u : kNever;
    unsigned long long s_e2e = 0, s_ttft = 0, s_tpot = 0;
    uint32_t last_fin = 0, n_ok = 0, n_rej = 0;

    const uint32_t n_t = (q.i_list + kTile - 1u) / kTile;
    for (uint32_t j0 = 0; j0 < n_t; j0 += kReplayTiles) {
        const uint32_t r0 = j0 * kTile, n = min(kReplayTiles * kTile, p.R - r0);
        __syncthreads();                                                            // the last stage's records were read
        for (uint32_t i = tid; i < n; i += kReplayListThreads) {
            const uint2 rq = p.req8[r0 + i];
            if constexpr (kTabled) {
                const uint2 cost = p.tab_pair[q.a + r0 + i];
                recs[i] = make_uint4(rq.x, rq.y >> 16, cost.x, cost.y);
            } else {
                recs[i] = rq;
            }
        }
        __syncthreads();
        for (uint32_t j = j0; j < min(j0 + kReplayTiles, n_t); ++j) {
        const staged_t* tile_recs = recs + (j - j0) * kTile;
        const size_t tile_at = (size_t)(live ? cb : 0u) * p.n_list_tiles + j;
        const uint32_t d = live ? p.desc[tile_at * (p.M + 1u) + m] : 0u;
        uint32_t count = d >> 16;
        const uint32_t first = d & 0xFFFFu;
        if ((first & 7u) != 0u || first + ((count + 7u) & ~7u) > p.tile_cap) count = 0u;   // never written that way
        const uint4* src = reinterpret_cast<const uint4*>(p.lists + tile_at * p.tile_cap + first);
        uint2* bins = p.bins + tile_at * p.tile_cap + first;                        // of this run; its padding reads "not served"
        for (uint32_t b = 0;; ++b) {
            const bool more = 8u * b < count;
            if (__ballot(more) == 0ull) break;
            uint4 e = make_uint4(0u, 0u, 0u, 0u);
            if (more) e = src[b];
            const uint32_t word[4] = {e.x, e.y, e.z, e.w};
            if (kBinsOut && with_hist && more && 8u * b + 8u > count) {             // the run's last block: its padding
#pragma unroll
                for (uint32_t k = 1; k < 8u; ++k)
                    if (8u * b + k >= count) bins[8u * b + k] = make_uint2(0u, 0u);
            }
#pragma unroll
            for (uint32_t k = 0; k < 8u; ++k) {
                const bool active = 8u * b + k < count;
                if (k != 0u && __ballot(active) == 0ull) break;
                const uint32_t rl = ((k & 1u) ? word[k >> 1] >> 16 : word[k >> 1]) & (kTile - 1u);
                const staged_t rq = tile_recs[rl];
                uint32_t prefill, tpot, out;
                if constexpr (kTabled) {
                    out = rq.y;
                    prefill = rq.z;
                    tpot = rq.w;
                } else {
                    const uint32_t prompt = rq.y & 0xFFFFu;
                    out = rq.y >> 16;
                    prefill = q.a + __umul24(q.b, prompt);                          // the host keeps all factors below 2^24
                    tpot = q.c + __umul24(q.d, (prompt + 1023u) >> 10);
                }
                const uint32_t dec = __umul24(out, tpot);
                const uint32_t start = max(max(rq.x, q.t_on), s[0]);
                const bool served = active && start < q.t_off;
                const uint32_t fin = start + prefill + dec;
                const uint32_t f = served ? fin : 0u;
#pragma unroll
                for (uint32_t i = 0; i + 1u < kSlots; ++i) s[i] = median3(s[i], f, s[i + 1u]);
                s[kSlots - 1u] = max(s[kSlots - 1u], f);
                if (served) {
                    const uint32_t ttft = start - rq.x + prefill;
                    const uint32_t e2e = ttft + dec;
                    s_ttft += ttft;
                    s_e2e += e2e;
                    s_tpot += tpot;
                    last_fin = max(last_fin, fin);
                    n_ok += (ttft <= p.slo_ttft && tpot <= p.slo_tpot) ? 1u : 0u;
                    if (kBinsOut && with_hist)
                        bins[8u * b + k] = make_uint2(hist_bin_u32(ttft) | (hist_bin_u32(e2e) << 12) | kBinServed,
                                                      hist_bin_u32(tpot));
                } else if (active) {
                    n_rej += 1u;                                                    // the replica is gone before it could start
                    if (kBinsOut && with_hist) bins[8u * b + k] = make_uint2(0u, 0u);
                }
            }
        }
        }
    }
    if (!live) return;
    // does the listed part leave the streamed part the room the host counted on?
    uint32_t flag = 0u;
    if (q.t_split != kNever) {
        uint32_t busy = 0u;
#pragma unroll
        for (uint32_t i = 0; i < kSlots; ++i) busy += (i < p.B && s[i] > q.t_split) ? 1u : 0u;
        if (busy > q.allow_busy) flag = kFlagFallback;
    }
    SplitPartial* sp = p.part + cb;
    if (s_e2e) atomicAdd(&sp->s_e2e, s_e2e);
    if (s_ttft) atomicAdd(&sp->s_ttft, s_ttft);
    if (s_tpot) atomicAdd(&sp->s_tpot, s_tpot);
    if (last_fin) atomicMax(&sp->last_fin, last_fin);
    if (n_ok) atomicAdd(&sp->n_ok, n_ok);
    if (n_rej) atomicAdd(&sp->n_rej, n_rej);
    if (flag) atomicOr(&sp->flags, flag);
}

// Merge: one record per candidate from its partial sums.  A candidate settled by penalty is written by one
// thread; one that the list replay handed back gets the pending mark (the general replay scores it next); for
// the others a workgroup takes the streamed requests' histograms from device memory, adds the bins the list replay
// left for every list position of the candidate (padding reads "not served") and goes through the usual
// block-wide reduction.
template <bool kHist16>
__global__ __launch_bounds__(kThreads) void k_merge_candidates(EvalParams p, SplitParams sp, ap_metrics* __restrict__ out,
                                                               uint32_t c0, uint32_t n_cand, PendingWord flags) {
    extern __shared__ __align__(16) unsigned char lds[];
    uint32_t* hist = reinterpret_cast<uint32_t*>(lds);
    unsigned long long* acc64 = reinterpret_cast<unsigned long long*>(lds + p.off_misc);
    uint32_t* acc32 = reinterpret_cast<uint32_t*>(lds + p.off_misc + 24);
    uint32_t* wtot = reinterpret_cast<uint32_t*>(lds + p.off_misc + 64);
    const uint32_t tid = threadIdx.x;
    // One workgroup per candidate that needs its histograms; the others are one thread's work each, so a
    // workgroup first settles a run of kThreads of them.
    for (uint32_t base = blockIdx.x * kThreads; base < n_cand; base += gridDim.x * kThreads) {
        const uint32_t cb = base + tid;
        if (cb < n_cand) {
            const SplitPartial part = sp.part[cb];
            if (part.flags & kFlagFallback) {
                unsigned long long* dst = reinterpret_cast<unsigned long long*>(&out[c0 + cb]);
#pragma unroll
                for (uint32_t i = 0; i < 8u; ++i) dst[i] = ~0ull;
                pending_raise(flags);
            } else if (part.flags & kFlagLazy) {
                const unsigned long long penalty = (unsigned long long)part.n_rej * p.penalty;
                const unsigned long long edge = hist_lower_edge(p.penalty_bin);
                ap_metrics mt;
                mt.sum_e2e_us = part.s_e2e + penalty;
                mt.sum_ttft_us = part.s_ttft + penalty;
                mt.sum_tpot_us = part.s_tpot + penalty;
                mt.makespan_us = part.last_fin;
                mt.p99_ttft_us = edge;
                mt.p99_tpot_us = edge;
                mt.p99_e2e_us = edge;
                mt.slo_ok = part.n_ok;
                mt.n_rejected = part.n_rej;
                out[c0 + cb] = mt;
            }
        }
    }
    for (uint32_t c = blockIdx.x; c < n_cand; c += gridDim.x) {
        const SplitPartial part = sp.part[c];                                       // the same for every thread
        if (part.flags & (kFlagFallback | kFlagLazy)) continue;
        const uint32_t* src = sp.hist + (size_t)c * sp.hist_words;
        const bool parked = (part.flags & kFlagNoStreamHist) == 0u;
        for (uint32_t i = tid; i < sp.hist_words; i += kThreads) hist[i] = parked ? src[i] : 0u;
        if (tid < 16u) reinterpret_cast<uint32_t*>(acc64)[tid] = 0u;
        __syncthreads();
        const size_t tiles_at = (size_t)c * sp.n_list_tiles;
        for (uint32_t j = 0; j < sp.n_list_tiles; ++j) {
            const uint32_t used = min(sp.desc[(tiles_at + j) * (sp.M + 1u) + sp.M], sp.tile_cap);
            const size_t at = (tiles_at + j) * sp.tile_cap;
            for (uint32_t i = tid; i < used; i += kThreads) {
                const uint2 word = sp.bins[at + i];
                if (word.x & kBinServed) {
                    hist_add<kHist16>(hist, 0u, word.x & 0xFFFu, 1u);
                    hist_add<kHist16>(hist, 1u, min(word.y, kBins - 1u), 1u);
                    hist_add<kHist16>(hist, 2u, (word.x >> 12) & 0xFFFu, 1u);
                }
            }
        }
        __syncthreads();
        const bool first_thread = tid == 0u;
        finish_candidate<kHist16>(p, hist, acc64, acc32, wtot, first_thread ? part.s_e2e : 0ull,
                                  first_thread ? part.s_ttft : 0ull, first_thread ? part.s_tpot : 0ull,
                                  first_thread ? part.last_fin : 0u, first_thread ? part.n_ok : 0u,
                                  first_thread ? part.n_rej : 0u, &out[c0 + c]);
        __syncthreads();
    }
}

}  // namespace

#endif  // AP_SPLIT_HPP
