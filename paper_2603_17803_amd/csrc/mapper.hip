// Request mapping (Section 6.1): merge the clusters activated by a group of selections, drop the
// DRAM-resident ones, and fill one bucket per SSD by sending each cluster -- in ascending
// (replication factor, cluster id) -- to its least-loaded replica.
//
// One wavefront per group.  The merge is an LDS bitmap (atomic-or per selected entry), compacted
// in ascending cluster id.  The greedy assignment is an inherently sequential chain over the
// distinct clusters, so the kernel is built around the length of one link: the per-item data
// (candidate-SSD mask, weight) is staged 64 items at a time in registers, one item per lane, and
// handed to the chain through v_readlane; lane d carries bucket d's load packed as
// (load << 6 | d), so one DPP min-reduction over the candidate lanes yields the least-loaded
// replica with ties to the lower SSD id, and only the compare-and-add of the winner stays on the
// dependent path.  Bucket positions are computed afterwards, in parallel, from the winners.
#include <type_traits>

#include "common.h"
#include "select_core.h"
#include "wave_ops.h"

namespace {

using waveops::low_lanes_min;
using waveops::lane_group_min;
using waveops::wave_excl_scan;

constexpr uint32_t INF32 = 0xffffffffu;

struct MapArgs {
    const int32_t* sel; int S; int H; int N; const int32_t* e2c; int Nc; const int32_t* replicas; int R; int D;
    const int32_t* weight; const uint32_t* resident; int32_t* q_off; int32_t* q_cluster; int32_t* q_load; int cap;
    uint32_t* dev_flags;
    int split_off;      // word offset of the 2 * cap words the split into independent sub-problems needs; 0 = no room, never split
    int piece;          // strided selections (the streams of a step, as the selection writes them): a group's S entries are
    int piece_stride;   // pieces of `piece` consecutive ids, `piece_stride` words apart; unused by the contiguous kernels
    int piece_shift;    // log2(piece) when it is a power of two (a shift instead of a division per entry), -1 otherwise
};

// Chain over items [0, m) in visiting order.  keybase = (load << 6) | lane.  On return assign[i]
// holds (ssd << 24) | position-in-bucket for every routed item and INF32 for unroutable ones;
// cnt is the bucket length of SSD `lane`.
//
// Items are staged 32 at a time, one per lane (lanes 0..31).  A single wave issues one instruction at a
// time, so a link of the chain costs its instruction count, not only its dependent path; what can be done
// per batch instead of per link is: the candidate masks are transposed once (SSD lane d gets the word whose
// bit j says "not a candidate of item j", D ballots per batch), so a link needs one signed bit-field extract
// for its mask, one v_readlane for its weight, and item numbers are literals (the batch is unrolled in
// groups of 8 behind uniform branches).  Per link then: extract, or, DPP min over the SSD lanes, compare,
// add, select, and two operations that set bit j of the winner's `won` word; bucket positions come from
// those words afterwards, off the chain.  The dependent path of a link matters as much as its length
// (every DPP step waits for its predecessor), hence the prepared keys below.
template <int STEPS>
__device__ __forceinline__ void greedy_chain_packed(uint32_t m, int lane, const uint32_t* order, const uint32_t* mask_lo,
                                                    const uint32_t* mask_hi, const uint32_t* wgt, uint32_t* assign,
                                                    uint32_t& keybase, uint32_t& cnt, int D, bool identity = false) {
    const uint32_t lane5 = (uint32_t)lane & 31u;
    for (uint32_t base = 0; base < m; base += 32) {
        const uint32_t n = min(32u, m - base);
        uint32_t it = 0, mlo = 0, mhi = 0, w6 = 0;
        if ((uint32_t)lane < n) {
            it = identity ? base + (uint32_t)lane : order[base + lane];     // identity: the visiting order is the list order, no look-up
            mlo = mask_lo[it];
            mhi = mask_hi[it];
            w6 = (wgt[it] << 6) & (0u - (uint32_t)((mlo | mhi) != 0u));   // an unroutable item adds no load (read with the masks, not after them)
        }
        uint32_t won = 0;
        // Slots past n hold an empty mask: every lane then "wins" with weight 0, which changes nothing,
        // so the unrolled groups of 8 need no per-item bound.
        if constexpr (STEPS <= 4) {
            uint32_t cand_t = 0;                               // bit j: this SSD lane is a candidate of item j
#pragma unroll
            for (int d = 0; d < (1 << STEPS); d += 4) {        // masks hold no bits at or beyond D
                const uint32_t b0 = (uint32_t)__ballot((mlo >> d) & 1u), b1 = (uint32_t)__ballot((mlo >> (d + 1)) & 1u);
                const uint32_t b2 = (uint32_t)__ballot((mlo >> (d + 2)) & 1u), b3 = (uint32_t)__ballot((mlo >> (d + 3)) & 1u);
                // lane d + i takes ballot i.  Literal lane numbers: no lane-select hazard; the wait covers "a vector
                // compare wrote the scalar register the next vector instruction reads" (2 wait states), which the
                // compiler cannot see into the statement to provide.
                asm("s_nop 1\n\tv_writelane_b32 %0, %1, %5\n\tv_writelane_b32 %0, %2, %6\n\tv_writelane_b32 %0, %3, %7\n\tv_writelane_b32 %0, %4, %8"
                    : "+v"(cand_t)
                    : "s"(b0), "s"(b1), "s"(b2), "s"(b3), "n"(d), "n"(d + 1), "n"(d + 2), "n"(d + 3));
            }
            const int32_t not_cand_t = (int32_t)~cand_t;
#pragma unroll
            for (uint32_t q = 0; q < 32; q += 8) {
                if (q < n) {
                    // The key of the next link is prepared for both outcomes of this one (the lane keeps its load or takes
                    // the weight) while the minimum is on its way, so that only the minimum, the compare and one select
                    // lie between two links.
                    uint32_t key = keybase | (uint32_t)((int32_t)((uint32_t)not_cand_t << (31u - q)) >> 31);
#pragma unroll
                    for (uint32_t u = 0; u < 8; ++u) {
                        const uint32_t j = q + u;
                        const uint32_t s_w6 = (uint32_t)__builtin_amdgcn_readlane((int)w6, (int)j);
                        uint32_t bumped = keybase + s_w6;
                        asm volatile("" : "+v"(bumped));                        // kept as a sum to select, not folded into select-then-add
                        uint32_t key_stay = 0, key_bump = 0;
                        if (u < 7) {
                            const uint32_t nc_next = (uint32_t)((int32_t)((uint32_t)not_cand_t << (31u - (j + 1))) >> 31);   // 0 or all ones
                            key_stay = keybase | nc_next;
                            key_bump = bumped | nc_next;
                            asm volatile("" : "+v"(key_stay), "+v"(key_bump));
                        }
                        const uint32_t best = lane_group_min<STEPS>(key);
                        const bool i_win = key == best;              // the winning SSD lane (every lane for an empty mask)
                        keybase = i_win ? bumped : keybase;
                        if (u < 7) key = i_win ? key_bump : key_stay;
                        won |= (uint32_t)i_win << j;
                    }
                }
            }
        } else {
            for (uint32_t q = 0; q < n; q += 8) {
#pragma unroll
                for (uint32_t u = 0; u < 8; ++u) {
                    const uint32_t j = q + u;
                    const uint32_t s_lo = (uint32_t)__builtin_amdgcn_readlane((int)mlo, (int)j);
                    const uint32_t s_w6 = (uint32_t)__builtin_amdgcn_readlane((int)w6, (int)j);
                    uint32_t bits = s_lo;
                    if (STEPS > 5) {
                        const uint32_t s_hi = (uint32_t)__builtin_amdgcn_readlane((int)mhi, (int)j);
                        bits = lane >= 32 ? s_hi : s_lo;
                    }
                    const uint32_t not_cand = ((bits >> lane5) & 1u) - 1u;      // 0 for a candidate SSD lane, all ones otherwise
                    const uint32_t bumped = keybase + s_w6;                     // off the dependent path
                    const uint32_t key = keybase | not_cand;
                    const uint32_t best = low_lanes_min<STEPS>(key);
                    const bool i_win = key == best;                  // the winning SSD lane (every lane for an empty mask)
                    keybase = i_win ? bumped : keybase;
                    won |= i_win ? (1u << j) : 0u;
                }
            }
        }
        // bucket positions of this chunk's items, in item order
        const bool routable = (mlo | mhi) != 0u;
        const uint32_t valid = (uint32_t)__ballot(routable);      // lanes >= 32 stage nothing, so this is a 32-bit item mask
        uint32_t my_assign = INF32;
        if constexpr (STEPS <= 4) {
            // item lane j: its SSD is the lane whose `won` word has bit j (for a routable item exactly one, below D);
            // that lane's word and bucket length then come by one lane gather each
            const uint32_t lanebit = 1u << lane5;
            uint32_t dj = 0;
#pragma unroll
            for (int d = 1; d < (1 << STEPS); ++d) {
                const uint32_t w_d = (uint32_t)__builtin_amdgcn_readlane((int)won, d);
                dj = (w_d & lanebit) ? (uint32_t)d : dj;
            }
            const uint32_t w_sel = (uint32_t)__builtin_amdgcn_ds_bpermute((int)(dj << 2), (int)won);
            const uint32_t c_sel = (uint32_t)__builtin_amdgcn_ds_bpermute((int)(dj << 2), (int)cnt);
            if (routable && lane < 32) my_assign = (dj << 24) | (c_sel + (uint32_t)__popc(w_sel & (lanebit - 1u) & valid));
        } else {
            for (int dsk = 0; dsk < D; ++dsk) {
                const uint32_t w_d = (uint32_t)__builtin_amdgcn_readlane((int)won, dsk);
                const uint32_t c_d = (uint32_t)__builtin_amdgcn_readlane((int)cnt, dsk);
                if (routable && lane < 32 && ((w_d >> lane) & 1u))
                    my_assign = ((uint32_t)dsk << 24) | (c_d + (uint32_t)__popc(w_d & ((1u << lane) - 1u) & valid));
            }
        }
        if ((uint32_t)lane < n) assign[it] = my_assign;
        cnt += __popc(won & valid);
    }
}

// Fallback for bucket loads that may exceed 2^26: loads are compared in full, ties resolved by ballot.
template <int STEPS>
__device__ __forceinline__ void greedy_chain_wide(uint32_t m, int lane, const uint32_t* order, const uint32_t* mask_lo,
                                                  const uint32_t* mask_hi, const uint32_t* wgt, uint32_t* assign,
                                                  uint32_t& load, uint32_t& cnt, bool identity = false) {
    for (uint32_t it = 0; it < m; ++it) {
        const uint32_t i = identity ? it : order[it];
        const uint64_t mask = ((uint64_t)mask_hi[i] << 32) | mask_lo[i];
        if (mask == 0) { if (lane == 0) assign[i] = INF32; continue; }
        const bool cand = (mask >> lane) & 1ull;
        const uint32_t key = cand ? load : INF32;
        const uint32_t best = low_lanes_min<STEPS>(key);
        const uint64_t tie = __ballot(cand && key == (uint32_t)__builtin_amdgcn_readfirstlane((int)best));
        const int winner = __ffsll((unsigned long long)tie) - 1;
        if (lane == winner) {
            assign[i] = ((uint32_t)winner << 24) | cnt;
            load += wgt[i];
            ++cnt;
        }
    }
}

// Chain of a sub-problem with exactly two SSDs, sa < sb (e.g. a replica pair of the round-robin placement with two
// replicas), or with the single SSD sa (sb < 0: no replication).  There is one comparison per link, so both loads live in scalar registers and a link is scalar work:
// compare, two selects, two adds (plus the bit that records the winner), where the general chain reduces over SSD lanes.
// Items come 64 at a time, one per lane.  An item with a single candidate needs no comparison: a run of such items is
// added up in parallel (they come first in the visiting order, which is by replication factor); a run of items with
// both candidates is walked link by link.  Same results as the general chain: ties go to the lower SSD.
__device__ __forceinline__ void greedy_chain_pair(uint32_t m, int lane, const uint32_t* order, const uint32_t* mask_lo,
                                                  const uint32_t* wgt, uint32_t* assign, uint32_t& keybase, uint32_t& cnt,
                                                  int sa, int sb) {
    const int sbr = sb >= 0 ? sb : sa;             // sb < 0: a sub-problem of the single SSD sa (no item has a second candidate)
    uint32_t la = (uint32_t)__builtin_amdgcn_readlane((int)keybase, sa) >> 6, lb = (uint32_t)__builtin_amdgcn_readlane((int)keybase, sbr) >> 6;
    uint32_t ca = (uint32_t)__builtin_amdgcn_readlane((int)cnt, sa), cb = (uint32_t)__builtin_amdgcn_readlane((int)cnt, sbr);
    for (uint32_t base = 0; base < m; base += 64) {
        const uint32_t n = min(64u, m - base);
        uint32_t it = 0, ml = 0, w = 0;
        if ((uint32_t)lane < n) {
            it = order[base + lane];
            ml = mask_lo[it];
            w = wgt[it];
        }
        const bool ha = (ml >> sa) & 1u, hb = sb >= 0 && ((ml >> sbr) & 1u);
        const uint64_t only_a = __ballot(ha && !hb), only_b = __ballot(!ha && hb), both = __ballot(ha && hb);
        const uint64_t single = only_a | only_b;
        const uint32_t w_both = (ha && hb) ? w : 0u;
        uint64_t to_b = only_b;
        uint32_t pos = 0;
        while (pos < n) {
            const uint64_t from = ~0ull << pos;                  // pos < 64
            // a run of items without a comparison (single candidate, or none): up to the next item with both
            const uint64_t nb = both & from;
            const uint32_t s_end = nb ? (uint32_t)__ffsll((unsigned long long)nb) - 1u : n;
            if (s_end > pos) {
                const uint64_t run = from & (s_end < 64u ? ~(~0ull << s_end) : ~0ull);
                if (single & run) {
                    const bool mine = (run >> lane) & 1ull;
                    uint32_t ta, tb;
                    (void)wave_excl_scan((mine && ha && !hb) ? w : 0u, &ta);
                    (void)wave_excl_scan((mine && hb && !ha) ? w : 0u, &tb);
                    la += ta;
                    lb += tb;
                }
            }
            // a run of items with both candidates: up to the next item without
            const uint64_t ns = ~both & (s_end < 64u ? ~0ull << s_end : 0ull);
            const uint32_t b_end = min(n, ns ? (uint32_t)__ffsll((unsigned long long)ns) - 1u : 64u);
            // A link in scalar arithmetic (loads stay below 2^26, so a sign is a comparison).
            if (s_end == 0u && b_end == n) {
                // The whole batch is one run (the common case: the items with a single candidate come first in the visiting
                // order).  The chain runs on the difference d = la - lb: SSD sb takes the item when d > 0 (equal loads: the
                // lower SSD), which lowers d by the weight; otherwise sa takes it and d rises.  Lane j of `dlog` keeps the
                // difference item j met (literal lane numbers: the batch is unrolled in groups of 8 behind uniform
                // branches; slots past n carry weight 0 and change nothing); the winners are read off it afterwards, and
                // the two loads follow from their sum and their difference.
                int32_t d = (int32_t)(la - lb);
                uint32_t dlog = 0u;
#pragma unroll
                for (uint32_t q = 0; q < 64; q += 8) {
                    if (q < n) {
                        int32_t s_w[8];                                      // the group's weights first: a link then never waits for its own
#pragma unroll
                        for (uint32_t u = 0; u < 8; ++u) s_w[u] = __builtin_amdgcn_readlane((int)w_both, (int)(q + u));
                        asm volatile("" : "+s"(s_w[0]), "+s"(s_w[1]), "+s"(s_w[2]), "+s"(s_w[3]), "+s"(s_w[4]), "+s"(s_w[5]), "+s"(s_w[6]), "+s"(s_w[7]));
#pragma unroll
                        for (uint32_t u = 0; u < 8; ++u) {
                            asm("v_writelane_b32 %0, %1, %2" : "+v"(dlog) : "s"(d), "n"(q + u));
                            int32_t lower = d - s_w[u], higher = d + s_w[u];   // both outcomes beside the comparison: two steps on the dependent path, not three
                            asm volatile("" : "+s"(lower), "+s"(higher));
                            d = d > 0 ? lower : higher;
                        }
                    }
                }
                to_b |= both & __ballot((int32_t)dlog > 0);
                uint32_t wrun;
                (void)wave_excl_scan(w_both, &wrun);
                const uint32_t sum = la + lb + wrun;            // below 2^27
                la = (uint32_t)((int32_t)sum + d) >> 1;
                lb = (uint32_t)((int32_t)sum - d) >> 1;
            } else {
                for (uint32_t j = s_end; j < b_end; ++j) {
                    const uint32_t s_w = (uint32_t)__builtin_amdgcn_readlane((int)w_both, (int)j);
                    const uint32_t pick_b = (uint32_t)((int32_t)(lb - la) >> 31);        // all ones: SSD sb
                    la += s_w & ~pick_b;
                    lb += s_w & pick_b;
                    to_b |= (uint64_t)(pick_b & 1u) << j;
                }
            }
            pos = b_end;
        }
        // bucket positions, in item order
        const uint64_t routed = single | both;
        const uint64_t to_a = routed & ~to_b;
        const uint64_t below = (1ull << lane) - 1ull;
        if ((uint32_t)lane < n) {
            uint32_t as = INF32;
            if ((routed >> lane) & 1ull)
                as = ((to_b >> lane) & 1ull) ? (((uint32_t)sb << 24) | (cb + (uint32_t)__popcll(to_b & below)))
                                             : (((uint32_t)sa << 24) | (ca + (uint32_t)__popcll(to_a & below)));
            assign[it] = as;
        }
        ca += (uint32_t)__popcll(to_a);
        cb += (uint32_t)__popcll(to_b);
    }
    if (lane == sa) { keybase = (la << 6) | (uint32_t)lane; cnt = ca; }
    if (lane == sb) { keybase = (lb << 6) | (uint32_t)lane; cnt = cb; }
}

__device__ __forceinline__ void run_chain_packed(int D, uint32_t m, int lane, const uint32_t* order, const uint32_t* mask_lo,
                                                 const uint32_t* mask_hi, const uint32_t* wgt, uint32_t* assign, uint32_t& keybase,
                                                 uint32_t& cnt, bool identity = false) {
    if (D <= 4) greedy_chain_packed<2>(m, lane, order, mask_lo, mask_hi, wgt, assign, keybase, cnt, D, identity);
    else if (D <= 8) greedy_chain_packed<3>(m, lane, order, mask_lo, mask_hi, wgt, assign, keybase, cnt, D, identity);
    else if (D <= 16) greedy_chain_packed<4>(m, lane, order, mask_lo, mask_hi, wgt, assign, keybase, cnt, D, identity);
    else greedy_chain_packed<6>(m, lane, order, mask_lo, mask_hi, wgt, assign, keybase, cnt, D, identity);
}

constexpr int MAP_THREADS = 256;
constexpr uint32_t MAP_SPLIT_MIN_ITEMS = 96;     // below this a single chain is shorter than finding the sub-problems

// Copies n words from global memory to LDS with batches of independent loads (all loads of a batch
// are in flight together, so a small table costs one memory round trip).  16-byte loads when the
// source allows it.
template <int NT>
__device__ __forceinline__ void stage_words(int32_t* __restrict__ dst, const int32_t* __restrict__ src, int n, int tid) {
    constexpr int BATCH = 8;
    if (((reinterpret_cast<uintptr_t>(src) & 15) == 0) && (n & 3) == 0) {
        const int n4 = n >> 2;
        const int4* s4 = reinterpret_cast<const int4*>(src);
        int4* d4 = reinterpret_cast<int4*>(dst);
        for (int base = 0; base < n4; base += BATCH * NT) {
            int4 v[BATCH];
#pragma unroll
            for (int u = 0; u < BATCH; ++u) {
                const int i = base + u * NT + tid;
                v[u] = (i < n4) ? s4[i] : make_int4(0, 0, 0, 0);
            }
#pragma unroll
            for (int u = 0; u < BATCH; ++u) {
                const int i = base + u * NT + tid;
                if (i < n4) d4[i] = v[u];
            }
        }
    } else {
        for (int base = 0; base < n; base += BATCH * NT) {
            int32_t v[BATCH];
#pragma unroll
            for (int u = 0; u < BATCH; ++u) {
                const int i = base + u * NT + tid;
                v[u] = (i < n) ? src[i] : 0;
            }
#pragma unroll
            for (int u = 0; u < BATCH; ++u) {
                const int i = base + u * NT + tid;
                if (i < n) dst[i] = v[u];
            }
        }
    }
}

// LDS layout shared by the stand-alone and the fused kernel.
constexpr int MAP_AUX_WORDS = 8 * 64;        // off, adj_lo, adj_hi, comp_of, seg_first, seg_cnt, pub_load, pub_cnt: 64 words each

struct MapLds {
    uint32_t *bitmap, *list, *mask_lo, *mask_hi, *wgt, *order, *assign, *order2, *comp_item, *off;
    uint32_t *adj_lo, *adj_hi, *comp_of, *seg_first, *seg_cnt, *pub_load, *pub_cnt;
    int32_t *s_e2c, *s_rep, *s_wgt;
    int nwords;
    __device__ __forceinline__ MapLds(uint32_t* smem, const MapArgs& a, int stage_e2c, int stage_tab) {
        nwords = (a.Nc + 31) / 32;
        bitmap = smem;
        list = bitmap + nwords;
        mask_lo = list + a.cap;
        mask_hi = mask_lo + a.cap;
        wgt = mask_hi + a.cap;
        order = wgt + a.cap;
        assign = order + a.cap;
        off = assign + a.cap;                 // MAP_AUX_WORDS words from here
        order2 = smem + a.split_off;          // visiting order regrouped by independent sub-problem (only when split_off != 0)
        comp_item = order2 + a.cap;           // sub-problem of every item
        adj_lo = off + 64;
        adj_hi = adj_lo + 64;
        comp_of = adj_hi + 64;
        seg_first = comp_of + 64;          // routed items by their lowest candidate SSD
        seg_cnt = seg_first + 64;
        pub_load = seg_cnt + 64;
        pub_cnt = pub_load + 64;
        s_e2c = reinterpret_cast<int32_t*>(smem + ((off + MAP_AUX_WORDS - smem + 3) & ~3));   // N words when staged (16-byte aligned)
        s_rep = s_e2c + (stage_e2c ? ((a.N + 3) & ~3) : 0);                // Nc*R words when staged
        s_wgt = s_rep + (stage_tab ? ((a.Nc * a.R + 3) & ~3) : 0);         // Nc words when staged
    }
};

// One group on a block of NT threads.  All waves cooperate on staging and on the merge; wave 0
// alone runs the compaction, the chain and the emission (the chain is a single-wave algorithm).
// When the head's lookup tables are small they are staged in LDS by one burst of independent loads,
// so that the kernel pays one memory round trip instead of three dependent ones (selection ->
// cluster of entry -> replica row).  PRESTAGED: the caller has already filled the staged tables,
// cleared the bitmap and synchronised, and `sel` points into LDS.
// BIG: the kernel is meant for long lists (thousands of merged picks, hundreds of clusters): the per-item pass and
// the SSD adjacency run on every thread and the merge marks bytes.  The short-list kernels leave that code out --
// it is not only unused there, its mere presence between the phases cost them 0.25 us per launch.
template <int NT, bool PRESTAGED, bool BIG, bool STRIDED = false>
__device__ __forceinline__ void map_group(const MapArgs& a, int64_t g, const int32_t* __restrict__ sel, uint32_t* smem,
                                          int stage_e2c, int stage_tab) {
    // position of the group's s-th entry behind `sel`
    auto at = [&](int s0) __attribute__((always_inline)) {
        if (!STRIDED) return s0;
        const int pc = a.piece_shift >= 0 ? s0 >> a.piece_shift : s0 / a.piece;
        return pc * a.piece_stride + (s0 - pc * a.piece);
    };
    const MapLds L(smem, a, stage_e2c, stage_tab);
    const int nwords = L.nwords;
    uint32_t *bitmap = L.bitmap, *list = L.list, *mask_lo = L.mask_lo, *mask_hi = L.mask_hi, *wgt = L.wgt, *order = L.order,
             *assign = L.assign, *off = L.off, *order2 = L.order2;
    int32_t *s_e2c = L.s_e2c, *s_rep = L.s_rep, *s_wgt = L.s_wgt;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    const int h = (int)(g % a.H);
    const int64_t cbase = (int64_t)h * a.Nc;
    uint32_t flags = 0;

    const int32_t* e2c = a.e2c + (size_t)h * a.N;
    constexpr int SEL_REGS = BIG ? 8 : 4;           // long lists: 8192 merged picks on 1024 threads are one burst of loads, not two round trips
    int32_t my_sel[SEL_REGS];
    if (!PRESTAGED) {
        // burst of independent loads: the selection into registers, the tables into LDS
#pragma unroll
        for (int r = 0; r < SEL_REGS; ++r) {
            const int s0 = tid + r * NT;
            my_sel[r] = (s0 < a.S) ? sel[at(s0)] : -1;
        }
        // Replica and weight tables of at most two resp. one 16-byte vector per thread travel through registers beside the
        // entry->cluster table: staged one after the other, each table waited for a memory round trip of its own.
        const int nrep = a.Nc * a.R;
        const int32_t* rep_src = a.replicas + cbase * a.R;
        const int32_t* wgt_src = a.weight ? a.weight + cbase : nullptr;
        const bool rep_fast = stage_tab && (nrep & 3) == 0 && (nrep >> 2) <= 2 * NT && (reinterpret_cast<uintptr_t>(rep_src) & 15) == 0;
        const bool wgt_fast = stage_tab && wgt_src && (a.Nc & 3) == 0 && (a.Nc >> 2) <= NT && (reinterpret_cast<uintptr_t>(wgt_src) & 15) == 0;
        int4 v_rep[2] = {make_int4(0, 0, 0, 0), make_int4(0, 0, 0, 0)}, v_wgt = make_int4(0, 0, 0, 0);
        if (rep_fast) {
#pragma unroll
            for (int u = 0; u < 2; ++u)
                if (tid + u * NT < (nrep >> 2)) v_rep[u] = reinterpret_cast<const int4*>(rep_src)[tid + u * NT];
        }
        if (wgt_fast && tid < (a.Nc >> 2)) v_wgt = reinterpret_cast<const int4*>(wgt_src)[tid];
        if (stage_tab) {
            if (!rep_fast) stage_words<NT>(s_rep, rep_src, nrep, tid);
            if (!wgt_src) { for (int i = tid; i < a.Nc; i += NT) s_wgt[i] = 1; }
            else if (!wgt_fast) stage_words<NT>(s_wgt, wgt_src, a.Nc, tid);
        }
        if (stage_e2c) stage_words<NT>(s_e2c, e2c, a.N, tid);
        if (rep_fast) {
#pragma unroll
            for (int u = 0; u < 2; ++u)
                if (tid + u * NT < (nrep >> 2)) reinterpret_cast<int4*>(s_rep)[tid + u * NT] = v_rep[u];
        }
        if (wgt_fast && tid < (a.Nc >> 2)) reinterpret_cast<int4*>(s_wgt)[tid] = v_wgt;
        for (int w = tid; w < nwords; w += NT) bitmap[w] = 0;
        __syncthreads();
    }

    // merge: one bit per activated, non-resident cluster.  In two steps per batch -- every entry's cluster first
    // (independent lookups, all in flight together), then the bits -- so that a batch costs one look-up latency,
    // not one per entry; -2 marks "nothing to set".
    // (selects, not branches: a branch per entry would put every look-up into a basic block of its own and
    // serialise the batch)
    // STAGED is a compile-time copy of stage_e2c: a run-time choice between the LDS and the memory copy of the
    // table turns the look-up into a flat load, whose wait also waits for the selection loads still in flight.
    auto cluster_of = [&](int32_t e, auto staged_tag) __attribute__((always_inline)) -> int32_t {
        constexpr bool STAGED = decltype(staged_tag)::value;
        const bool e_ok = (uint32_t)e < (uint32_t)a.N;                     // -1 is padding of a ragged selection, anything else out of range is flagged
        flags |= (!e_ok && e != -1) ? SWARM_DEV_BAD_ENTRY : 0u;
        const int32_t ee = e_ok ? e : 0;
        const int32_t c = STAGED ? s_e2c[ee] : e2c[ee];
        const bool c_ok = (uint32_t)c < (uint32_t)a.Nc;
        flags |= (e_ok && !c_ok) ? SWARM_DEV_BAD_CLUSTER : 0u;
        return (e_ok && c_ok) ? c : -2;
    };
    // Long selections over few clusters (many streams merged) would send thousands of LDS atomics to a handful of
    // bitmap words; they mark one BYTE per cluster with plain stores instead (equal values, so collisions are
    // harmless) and the bytes are folded into the bitmap afterwards.  The byte map borrows the room of the split
    // arrays, which are not in use yet.
    const bool byte_marks = BIG && !PRESTAGED && a.split_off != 0 && a.S >= 2048 && (size_t)a.cap * 8 >= (size_t)a.Nc + 64;
    uint8_t* marks = reinterpret_cast<uint8_t*>(order2);
    if (byte_marks) {
        for (int i = tid; i < (a.Nc + 63) / 64 * 16; i += NT) reinterpret_cast<uint32_t*>(marks)[i] = 0u;
        __syncthreads();
    }
    auto set_bit = [&](int32_t c) __attribute__((always_inline)) {
        if (c < 0) return;
        if (a.resident) {
            const int64_t gc = cbase + c;
            if ((a.resident[gc >> 5] >> (gc & 31)) & 1u) return;
        }
        if (byte_marks) marks[c] = 1;
        else atomicOr(&bitmap[c >> 5], 1u << (c & 31));
    };
    auto merge_all = [&](auto staged_tag) __attribute__((always_inline)) {
        if (PRESTAGED) {                             // the selection is in LDS: nothing to batch
            for (int s0 = tid; s0 < a.S; s0 += NT) {
                const int32_t e = sel[s0];
                if (e == -1) continue;
                if (e < 0 || e >= a.N) { flags |= SWARM_DEV_BAD_ENTRY; continue; }
                const int32_t c = decltype(staged_tag)::value ? s_e2c[e] : e2c[e];
                if (c < 0 || c >= a.Nc) { flags |= SWARM_DEV_BAD_CLUSTER; continue; }
                if (a.resident) {
                    const int64_t gc = cbase + c;
                    if ((a.resident[gc >> 5] >> (gc & 31)) & 1u) continue;
                }
                atomicOr(&bitmap[c >> 5], 1u << (c & 31));
            }
            return;
        }
        {
            int32_t c[SEL_REGS];
#pragma unroll
            for (int r = 0; r < SEL_REGS; ++r) c[r] = (tid + r * NT < a.S) ? cluster_of(my_sel[r], staged_tag) : -2;
#pragma unroll
            for (int r = 0; r < SEL_REGS; ++r) set_bit(c[r]);
        }
        // long selections (many streams merged): the rest in batches of independent loads
        constexpr int MB = 8;
        for (int s0 = tid + SEL_REGS * NT; s0 < a.S; s0 += MB * NT) {
            int32_t e[MB], c[MB];
#pragma unroll
            for (int u = 0; u < MB; ++u) e[u] = (s0 + u * NT < a.S) ? sel[at(s0 + u * NT)] : -1;
#pragma unroll
            for (int u = 0; u < MB; ++u) c[u] = cluster_of(e[u], staged_tag);
#pragma unroll
            for (int u = 0; u < MB; ++u) set_bit(c[u]);
        }
    };
    if (stage_e2c) merge_all(std::true_type{});
    else merge_all(std::false_type{});
    __syncthreads();
    if (byte_marks) {
        for (int base = wave * 64; base < a.Nc; base += NT) {            // 64 clusters per wave and pass: two bitmap words
            const uint64_t set = __ballot(marks[base + lane] != 0);      // bytes past Nc were cleared and are never marked
            if (lane == 0) {
                bitmap[base >> 5] = (uint32_t)set;
                if ((base >> 5) + 1 < nwords) bitmap[(base >> 5) + 1] = (uint32_t)(set >> 32);
            }
        }
        __syncthreads();
    }

    // Every wave counts the merged clusters (a popcount of the bitmap).  Few of them: wave 0 does all the rest
    // alone, as one chain.  Many: wave 0 compacts, orders and looks for independent sub-problems, whose chains
    // then run side by side on the other waves; all waves meet at the barriers in between (the decision is
    // the same in every wave, so either all of them go to the barriers or none).
    constexpr bool SPLIT = BIG || !PRESTAGED;        // the fused short-list kernel (one step's selection) leaves the split out
    uint32_t m_all = 0;
    if (SPLIT) {
        for (int w0 = 0; w0 < nwords; w0 += 64) m_all += (w0 + lane < nwords) ? __popc(bitmap[w0 + lane]) : 0;
        uint32_t total;
        (void)wave_excl_scan(m_all, &total);
        m_all = min(total, (uint32_t)a.cap);
    }
    const bool try_split = SPLIT && NT > 64 && a.split_off != 0 && m_all >= MAP_SPLIT_MIN_ITEMS;
    if (wave != 0 && !try_split) {
        if (flags) atomicOr(a.dev_flags, flags);
        return;
    }
    uint32_t m = 0, load = 0, cnt = 0, wsum = 0;
    const int D = a.D;
    // Long lists: every thread places the cluster of its own bitmap bit (the words' popcounts are scanned by every wave
    // for itself: lane j = word j), instead of wave 0 walking the bitmap alone.
    const bool par_compact = BIG && try_split && nwords <= 64;
    uint32_t m_par = 0;
    if (par_compact) {
        const uint32_t wexcl = wave_excl_scan(lane < nwords ? (uint32_t)__popc(bitmap[lane]) : 0u, &m_par);
        for (int b0 = 0; b0 < nwords * 32; b0 += NT) {
            const int bit = b0 + tid, w = bit >> 5;
            const uint32_t word = w < nwords ? bitmap[w] : 0u;
            const uint32_t before = (uint32_t)__shfl((int)wexcl, w & 63, 64);
            if ((word >> (bit & 31)) & 1u) {
                const uint32_t pos = before + (uint32_t)__popc(word & ((1u << (bit & 31)) - 1u));
                if (pos < (uint32_t)a.cap) list[pos] = (uint32_t)bit;
            }
        }
    }
    if (wave == 0) {
    // compaction in ascending cluster id; a lane takes a slice of 8, 16 or 32 bits, the narrowest that still puts
    // the whole bitmap on the 64 lanes at once, so that a densely set, short bitmap is not walked by a few lanes
    const int pw_shift = nwords <= 16 ? 2 : nwords <= 32 ? 1 : 0;     // log2 of the slices per word
    const int sbits = 32 >> pw_shift, nslices = nwords << pw_shift;   // slice width: 8, 16 or 32 bits
    m = m_par;
    for (int s0 = 0; s0 < (par_compact ? 0 : nslices); s0 += 64) {
        const int sl = s0 + lane;
        const int w = sl >> pw_shift, sh = (sl & ((1 << pw_shift) - 1)) * sbits;
        uint32_t bits = (sl < nslices) ? ((bitmap[w] >> sh) & (sbits == 32 ? 0xffffffffu : (1u << sbits) - 1u)) : 0u;
        uint32_t total;
        uint32_t pos = m + wave_excl_scan(__popc(bits), &total);
        while (bits) {
            const int bit = __ffs(bits) - 1;
            bits &= bits - 1;
            if (pos < (uint32_t)a.cap) list[pos] = (uint32_t)(w * 32 + sh + bit);
            ++pos;
        }
        m += total;
    }
    if (__builtin_expect(m > (uint32_t)a.cap, 0)) { flags |= SWARM_DEV_CAP; m = a.cap; }
    if (BIG && try_split) {                          // what the other waves need for their share of the per-item pass
        if (lane == 0) { off[1] = m; off[2] = INF32; off[3] = 0u; off[4] = 0u; }
        L.adj_lo[lane] = 0u;
        L.adj_hi[lane] = 0u;
        L.seg_cnt[lane] = 0u;
        L.seg_first[lane] = 0u;
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
    }   // wave 0

    // per item: candidate SSD mask, weight, replication factor -- by wave 0 alone for a short list, by every thread
    // for a long one (which also gathers, per SSD, the union of the candidate masks that contain it)
    uint32_t rf_min = INF32, rf_max = 0;
    // TAB is a compile-time copy of stage_tab (a run-time choice between the LDS and the memory copy of a table
    // makes its look-ups flat loads); the replica slots are read four at a time, all in flight together (the index
    // is clamped: a slot read twice sets the same bit twice).
    auto item = [&](uint32_t i, auto tab_tag) __attribute__((always_inline)) {
        constexpr bool TAB = decltype(tab_tag)::value;
        const uint32_t c = list[i];
        const int64_t gc = cbase + c;
        uint64_t mask = 0;
        const int R = a.R;
        for (int r0 = 0; r0 < R; r0 += 4) {
            int32_t dsk[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int r = min(r0 + u, R - 1);
                dsk[u] = TAB ? s_rep[c * R + r] : a.replicas[gc * R + r];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {                         // selects, not branches: one basic block for the four slots
                flags |= (dsk[u] >= a.D) ? SWARM_DEV_BAD_SSD : 0u;
                mask |= ((uint32_t)dsk[u] < (uint32_t)a.D) ? (1ull << (dsk[u] & 63)) : 0ull;      // negative: an unused slot
            }
        }
        if (mask == 0) flags |= SWARM_DEV_BAD_SSD;
        mask_lo[i] = (uint32_t)mask;
        mask_hi[i] = (uint32_t)(mask >> 32);
        const int32_t wraw = TAB ? s_wgt[c] : (a.weight ? a.weight[gc] : 1);
        const uint32_t wv = (uint32_t)max(wraw, 0);
        wgt[i] = wv;
        wsum = min(wsum + min(wv, 1u << 26), 1u << 26);       // saturating: only "below 2^26" matters
        const uint32_t rf = __popcll(mask);
        order[i] = rf;                               // replication factor for now
        assign[i] = INF32;
        rf_min = min(rf_min, rf);
        rf_max = max(rf_max, rf);
        return mask;
    };
    auto reduce_wave = [&]() __attribute__((always_inline)) {
        rf_min = waveops::wave_min_u32(rf_min);
        rf_max = ~waveops::wave_min_u32(~rf_max);
        const bool any_big = __ballot(wsum >= (1u << 26)) != 0ull;
        uint32_t total;
        (void)wave_excl_scan(min(wsum, (1u << 26) - 1u), &total);     // <= 64 * (2^26 - 1): no wrap
        wsum = any_big ? (1u << 26) : min(total, 1u << 26);
    };
    if (BIG && try_split) {
        __syncthreads();
        const uint32_t mm = off[1];
        for (uint32_t i = tid; i < mm; i += NT) {
            uint64_t bits = stage_tab ? item(i, std::true_type{}) : item(i, std::false_type{});
            const uint32_t lo = (uint32_t)bits, hi = (uint32_t)(bits >> 32);
            if (bits) atomicAdd(&L.seg_first[__ffsll((unsigned long long)bits) - 1], 1u);
            while (bits) {
                const int d = __ffsll((unsigned long long)bits) - 1;
                bits &= bits - 1;
                if (lo) atomicOr(&L.adj_lo[d], lo);
                if (hi) atomicOr(&L.adj_hi[d], hi);
            }
        }
        reduce_wave();
        if (lane == 0) {                             // at most 16 waves x 2^26: no wrap
            atomicMin(&off[2], rf_min);
            atomicMax(&off[3], rf_max);
            atomicAdd(&off[4], wsum);
        }
        __syncthreads();
    }
    if (wave == 0) {
    if (BIG && try_split) {
        rf_min = off[2];
        rf_max = off[3];
        wsum = min(off[4], 1u << 26);
    } else {
        if (stage_tab) { for (uint32_t i = lane; i < m; i += 64) (void)item(i, std::true_type{}); }
        else { for (uint32_t i = lane; i < m; i += 64) (void)item(i, std::false_type{}); }
        reduce_wave();
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");

    // visiting order: stable by replication factor (identity when all factors agree)
    const bool identity = m > 0 && rf_min == rf_max;
    if (lane == 0) off[5] = identity ? 1u : 0u;
    if (__builtin_expect(identity, 1)) {
        // the list order is the visiting order: the chains and the split read it without a look-up, the table stays unwritten
    } else if (m > 0) {
        uint32_t* rfv = assign;                      // assign is rewritten below, before the chain runs
        for (uint32_t i = lane; i < m; i += 64) rfv[i] = order[i];
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
        uint32_t outpos = 0;
        for (uint32_t v = rf_min; v <= rf_max; ++v) {
            for (uint32_t i0 = 0; i0 < m; i0 += 64) {
                const uint32_t i = i0 + lane;
                const bool hit = (i < m) && (rfv[i] == v);
                const uint64_t b = __ballot(hit);
                if (hit) order[outpos + __popcll(b & ((1ull << lane) - 1ull))] = i;
                outpos += __popcll(b);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
        for (uint32_t i = lane; i < m; i += 64) assign[i] = INF32;
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");

    // Independent sub-problems: two SSDs interact only through an item that has both as candidates, so the
    // connected components of "share a routed item" never meet in a comparison and their chains can run side
    // by side, each in the visiting order of its own items (an SSD's bucket is filled by one component only,
    // so bucket positions are unchanged).  Lane d holds the set of SSDs reachable from d; Warshall's closure
    // by rows; a component is named by its lowest SSD.
    uint32_t ncomp = 1;
    if (try_split && wsum < (1u << 26)) {
        if (!BIG) {                                  // the adjacency was not gathered with the per-item pass
            L.adj_lo[lane] = 0u;
            L.adj_hi[lane] = 0u;
            L.seg_cnt[lane] = 0u;
            L.seg_first[lane] = 0u;
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
            for (uint32_t i = lane; i < m; i += 64) {
                const uint32_t lo = mask_lo[i], hi = mask_hi[i];
                uint64_t bits = ((uint64_t)hi << 32) | lo;
                if (bits) atomicAdd(&L.seg_first[__ffsll((unsigned long long)bits) - 1], 1u);
                while (bits) {
                    const int d = __ffsll((unsigned long long)bits) - 1;
                    bits &= bits - 1;
                    if (lo) atomicOr(&L.adj_lo[d], lo);
                    if (hi) atomicOr(&L.adj_hi[d], hi);
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
        }
        uint64_t reach = ((uint64_t)L.adj_hi[lane] << 32) | L.adj_lo[lane];
        const bool active = reach != 0ull;           // some routed item has SSD `lane` as a candidate (then reach holds lane itself)
        for (int kk = 0; kk < D; ++kk) {
            const uint64_t rk = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(reach >> 32), kk) << 32) |
                                (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)reach, kk);
            if ((reach >> kk) & 1ull) reach |= rk;
        }
        const int rep = active ? __ffsll((unsigned long long)reach) - 1 : 64;
        const uint64_t reps = __ballot(active && rep == lane);
        ncomp = (uint32_t)__popcll(reps);
        const uint32_t my_comp = active ? (uint32_t)__popcll(reps & ((1ull << rep) - 1ull)) : 0xffu;
        L.comp_of[lane] = my_comp;
        // an item belongs to the sub-problem of its lowest candidate SSD: the sub-problems' sizes from the per-SSD counts
        if (active && L.seg_first[lane]) atomicAdd(&L.seg_cnt[my_comp], L.seg_first[lane]);
    }
    if (lane == 0) off[0] = ncomp;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
    if (ncomp <= 1) {
        // greedy least-loaded assignment, one chain
        if (__builtin_expect(wsum < (1u << 26), 1)) {
            uint32_t keybase = (uint32_t)lane;
            run_chain_packed(D, m, lane, order, mask_lo, mask_hi, wgt, assign, keybase, cnt, identity);
            load = keybase >> 6;
        } else {
            if (D <= 16) greedy_chain_wide<4>(m, lane, order, mask_lo, mask_hi, wgt, assign, load, cnt, identity);
            else greedy_chain_wide<6>(m, lane, order, mask_lo, mask_hi, wgt, assign, load, cnt, identity);
        }
    }
    if (lane == 0) off[1] = m;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
    }   // wave 0
    uint32_t ncomp = 1;
    if (try_split) {
        __syncthreads();
        ncomp = off[0];
        if (ncomp > 1) {
            const uint32_t mm = off[1];
            const bool identity = off[5] != 0u;            // the visiting order is the list order: no look-up
            // component c on wave c mod (number of waves): the wave gathers the component's items in visiting
            // order (stable), then runs their chain; a wave that gets several components runs them one after the
            // other on the same registers (their SSDs are disjoint)
            constexpr uint32_t NW = NT / 64;
            uint32_t routed;
            const uint32_t seg = wave_excl_scan(L.seg_cnt[lane], &routed);      // lanes >= ncomp hold 0
            uint32_t keybase = (uint32_t)lane, mycnt = 0;
            for (uint32_t c = (uint32_t)wave; c < ncomp; c += NW) {
                const uint32_t base = (uint32_t)__builtin_amdgcn_readlane((int)seg, (int)c);
                const uint64_t ssds = __ballot(lane < D && L.comp_of[lane] == c);         // the component's SSDs
                const uint32_t ssds_lo = (uint32_t)ssds, ssds_hi = (uint32_t)(ssds >> 32);
                uint32_t run = 0;
                for (uint32_t i0 = 0; i0 < mm; i0 += 256) {          // four batches of look-ups in flight together
                    uint32_t it[4], ml[4], mh[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const uint32_t i = i0 + u * 64 + lane;
                        it[u] = i < mm ? (identity ? i : order[i]) : 0u;
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const bool in = i0 + u * 64 + lane < mm;
                        ml[u] = in ? mask_lo[it[u]] : 0u;
                        mh[u] = (in && D > 32) ? mask_hi[it[u]] : 0u;
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        // an item's candidates all lie in one sub-problem: any of them tells which
                        const bool hit = ((ml[u] & ssds_lo) | (mh[u] & ssds_hi)) != 0u;
                        const uint64_t b = __ballot(hit);
                        if (hit) order2[base + run + (uint32_t)__popcll(b & ((1ull << lane) - 1ull))] = it[u];
                        run += (uint32_t)__popcll(b);
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
                if (D <= 32 && __popcll(ssds) <= 2 && ssds != 0ull) {
                    const int sa = __ffsll((unsigned long long)ssds) - 1, sb = 63 - __clzll((unsigned long long)ssds);
                    greedy_chain_pair(run, lane, order2 + base, mask_lo, wgt, assign, keybase, mycnt, sa, sb != sa ? sb : -1);
                } else {
                    run_chain_packed(D, run, lane, order2 + base, mask_lo, mask_hi, wgt, assign, keybase, mycnt);
                }
            }
            if (lane < D) {
                const uint32_t c = L.comp_of[lane];
                if (c != 0xffu && c % NW == (uint32_t)wave) {
                    L.pub_load[lane] = keybase >> 6;
                    L.pub_cnt[lane] = mycnt;
                }
            }
        }
        __syncthreads();
    }
    // Bucket offsets are single-wave work; the scatter of the queues is per-item work, which the long-list kernels
    // leave to all their waves when those are still here (they are after a split into sub-problems).
    const bool all_emit = BIG && try_split;
    if (wave != 0 && !all_emit) {
        if (flags) atomicOr(a.dev_flags, flags);
        return;
    }
    uint32_t total = 0;
    if (wave == 0) {
        if (ncomp > 1) {
            const bool active = lane < D && L.comp_of[lane] != 0xffu;
            load = active ? L.pub_load[lane] : 0u;
            cnt = active ? L.pub_cnt[lane] : 0u;
        }
        // buckets SSD-major, insertion order inside a bucket
        const uint32_t my_off = wave_excl_scan(lane < D ? cnt : 0u, &total);
        off[lane] = my_off;
        int32_t* q_off = a.q_off + g * (D + 1);
        if (lane < D) {
            q_off[lane] = (int32_t)my_off;
            a.q_load[g * D + lane] = (int32_t)load;
        }
        if (lane == 0) {
            q_off[D] = (int32_t)total;
            if (all_emit) { L.seg_cnt[0] = total; L.seg_cnt[1] = m; }      // the sub-problems' sizes have been read
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
    }
    uint32_t m_emit = m;
    if (all_emit) {
        __syncthreads();
        total = L.seg_cnt[0];
        m_emit = L.seg_cnt[1];
    }
    const uint32_t first = all_emit ? (uint32_t)tid : (uint32_t)lane, step = all_emit ? (uint32_t)NT : 64u;
    int32_t* qc = a.q_cluster + g * a.cap;
    for (uint32_t i = first; i < m_emit; i += step) {
        const uint32_t as = assign[i];
        if (as != INF32) qc[off[as >> 24] + (as & 0xffffffu)] = (int32_t)list[i];
    }
    for (uint32_t p = total + first; p < (uint32_t)a.cap; p += step) qc[p] = -1;

    if (flags) atomicOr(a.dev_flags, flags);
}

// NT = 256 for a step's selection; 1024 for long merged selections, whose merge is plain per-entry work that
// scales with the number of threads.
// STRIDED: group g = (step g / H, head g % H) merges the B streams of that step out of selections laid out
// [step][stream][head][k], the layout the selection step writes.
template <int NT, bool STRIDED = false>
__global__ __launch_bounds__(NT) void map_requests_kernel(MapArgs a, int stage_e2c, int stage_tab) {
    extern __shared__ __attribute__((aligned(16))) uint32_t smem[];
    const int64_t g = blockIdx.x;
    const int32_t* sel = STRIDED ? a.sel + (g / a.H) * (int64_t)a.S * a.H + (g % a.H) * a.piece : a.sel + g * a.S;
    map_group<NT, false, (NT > 256), STRIDED>(a, g, sel, smem, stage_e2c, stage_tab);
}

// Selection and request mapping of one decode step of a single stream in one kernel: block h selects
// the k entries of head h (selcore::block_select, into LDS), writes them out, and maps them.  The
// lookup tables of the mapping do not depend on the selection: their loads are issued first and are
// in flight while the selection runs.  Per thread: up to 2 x 16 bytes of the entry->cluster table,
// 16 bytes of the replica table and 16 bytes of the weights (the host stages a table only if it fits
// that and is 16-byte aligned).
// CAND: second stage of the sliced selection of a long row -- the keys are the scores of the M listed winners of
// the row's slices (ascending entry id), and the selected list positions are turned back into entry ids.
template <int IPT, bool CAND, int NT = selcore::NT>
__global__ __launch_bounds__(NT) void select_map_kernel(const float* __restrict__ scores, int N, int k,
                                                        int32_t* __restrict__ out_idx, MapArgs a, int stage_e2c,
                                                        int stage_tab, int sel_off, const int32_t* __restrict__ cand,
                                                        int cand_stride, int M) {
    __shared__ selcore::SmemT<NT> sm;
    extern __shared__ __attribute__((aligned(16))) uint32_t smem[];
    const int tid = threadIdx.x;
    const int h = blockIdx.x;                                 // one stream: group = head
    const int64_t cbase = (int64_t)h * a.Nc;
    const MapLds L(smem, a, stage_e2c, stage_tab);

    // the scores first (the selection waits for them), then the tables (needed only after it)
    int32_t* sel_lds = reinterpret_cast<int32_t*>(smem + sel_off);
    uint32_t key[IPT];
    const int32_t* c = CAND ? cand + (size_t)h * cand_stride : nullptr;
    if (CAND) {
        const float* srow = scores + (size_t)h * N;
        const int base = tid * IPT;
#pragma unroll
        for (int e = 0; e < IPT; ++e) key[e] = (base + e < M) ? selcore::order_key(srow[c[base + e]]) : 0u;
    } else {
        selcore::load_keys<IPT>(scores + (size_t)h * N, N, key);
    }
    int4 r_e2c[2] = {make_int4(0, 0, 0, 0), make_int4(0, 0, 0, 0)}, r_rep = make_int4(0, 0, 0, 0), r_wgt = make_int4(0, 0, 0, 0);
    const int n4_e2c = a.N >> 2, n4_rep = (a.Nc * a.R) >> 2, n4_wgt = a.Nc >> 2;
    if (stage_e2c) {
        const int4* src = reinterpret_cast<const int4*>(a.e2c + (size_t)h * a.N);
#pragma unroll
        for (int u = 0; u < 2; ++u)
            if (tid + u * NT < n4_e2c) r_e2c[u] = src[tid + u * NT];
    }
    if (stage_tab) {
        if (tid < n4_rep) r_rep = reinterpret_cast<const int4*>(a.replicas + cbase * a.R)[tid];
        if (a.weight && tid < n4_wgt) r_wgt = reinterpret_cast<const int4*>(a.weight + cbase)[tid];
    }
    for (int w = tid; w < L.nwords; w += NT) L.bitmap[w] = 0;

    selcore::block_select<IPT, NT>(key, CAND ? M : N, k, sel_lds, sm);
    if (CAND) {
        __syncthreads();
        for (int i = tid; i < k; i += NT) sel_lds[i] = c[sel_lds[i]];
    }

    if (stage_e2c) {
#pragma unroll
        for (int u = 0; u < 2; ++u)
            if (tid + u * NT < n4_e2c) reinterpret_cast<int4*>(L.s_e2c)[tid + u * NT] = r_e2c[u];
    }
    if (stage_tab) {
        if (tid < n4_rep) reinterpret_cast<int4*>(L.s_rep)[tid] = r_rep;
        if (a.weight) { if (tid < n4_wgt) reinterpret_cast<int4*>(L.s_wgt)[tid] = r_wgt; }
        else for (int i = tid; i < a.Nc; i += NT) L.s_wgt[i] = 1;
    }
    __syncthreads();
    for (int i = tid; i < k; i += NT) out_idx[(size_t)h * k + i] = sel_lds[i];
    map_group<NT, true, CAND>(a, h, sel_lds, smem, stage_e2c, stage_tab);
}

}  // namespace

size_t map_lds_base_bytes(int Nc, int cap) { return ((size_t)(Nc + 31) / 32 + (size_t)cap * 6 + MAP_AUX_WORDS) * 4; }

// piece > 0: strided selections (see map_requests_kernel), S = streams x piece.
swarm_status launch_map(swarm_ctx* ctx, const int32_t* sel, int64_t groups, int S, int H, int N, const int32_t* e2c,
                        int Nc, const int32_t* replicas, int R, int D, const int32_t* weight,
                        const uint32_t* resident, int32_t* q_off, int32_t* q_cluster, int32_t* q_load, int cap, int piece) {
    MapArgs a{sel, S, H, N, e2c, Nc, replicas, R, D, weight, resident, q_off, q_cluster, q_load, cap, ctx->dev_flags, 0, piece, H * piece,
              (piece > 0 && (piece & (piece - 1)) == 0) ? __builtin_ctz((unsigned)piece) : -1};
    size_t lds = map_lds_base_bytes(Nc, cap);
    const size_t budget = 64u * 1024u;
    int stage_tab = 0, stage_e2c = 0;
    const size_t tab_bytes = ((size_t)Nc * R + 3) / 4 * 16 + ((size_t)Nc + 3) / 4 * 16, e2c_bytes = ((size_t)N + 3) / 4 * 16;
    lds = (lds + 15) / 16 * 16;
    if (lds + tab_bytes <= budget) { stage_tab = 1; lds += tab_bytes; }
    if (lds + e2c_bytes <= budget) { stage_e2c = 1; lds += e2c_bytes; }
    if (lds + (size_t)cap * 8 <= budget) { a.split_off = (int)(lds / 4); lds += (size_t)cap * 8; }
    if (piece > 0 && S >= 2048)
        hipLaunchKernelGGL((map_requests_kernel<1024, true>), dim3((unsigned)groups), dim3(1024), lds, ctx->stream, a, stage_e2c, stage_tab);
    else if (piece > 0)
        hipLaunchKernelGGL((map_requests_kernel<MAP_THREADS, true>), dim3((unsigned)groups), dim3(MAP_THREADS), lds, ctx->stream, a,
                           stage_e2c, stage_tab);
    else if (S >= 2048)
        hipLaunchKernelGGL(map_requests_kernel<1024>, dim3((unsigned)groups), dim3(1024), lds, ctx->stream, a, stage_e2c, stage_tab);
    else
        hipLaunchKernelGGL(map_requests_kernel<MAP_THREADS>, dim3((unsigned)groups), dim3(MAP_THREADS), lds, ctx->stream, a, stage_e2c,
                           stage_tab);
    return swarm_check_launch(ctx, "map_requests_kernel");
}

// Fused selection + mapping for one stream (groups = H, S = k).  *launched tells whether the shapes fit
// the fused kernel; when they do not, nothing is enqueued and the caller launches the two kernels
// separately.
swarm_status launch_select_map(swarm_ctx* ctx, const float* scores, int H, int N, int k, int32_t* out_idx,
                               const int32_t* e2c, int Nc, const int32_t* replicas, int R, int D, const int32_t* weight,
                               const uint32_t* resident, int32_t* q_off, int32_t* q_cluster, int32_t* q_load, int cap,
                               bool* launched) {
    *launched = false;
    const bool sliced = select_uses_slices(H, N, k);       // long rows: the slices' winners first, their selection fused with the mapping
    // short rows select with smaller blocks, four scores per thread (see launch_select)
    const int NT = sliced ? selcore::NT : N <= 4 * 256 ? 256 : N <= 4 * 512 ? 512 : selcore::NT;
    if (N > 64 * NT && !sliced) return SWARM_OK;
    MapArgs a{nullptr, k, H, N, e2c, Nc, replicas, R, D, weight, resident, q_off, q_cluster, q_load, cap, ctx->dev_flags, 0, 0, 0, -1};
    size_t lds = map_lds_base_bytes(Nc, cap);
    const size_t budget = 64u * 1024u;                     // dynamic part; the selection's static 12.6 KiB come on top
    lds = (lds + 15) / 16 * 16;
    int stage_tab = 0, stage_e2c = 0;
    const size_t tab_bytes = ((size_t)Nc * R + 3) / 4 * 16 + ((size_t)Nc + 3) / 4 * 16, e2c_bytes = ((size_t)N + 3) / 4 * 16;
    const bool tab_regs = (Nc * R) % 4 == 0 && Nc % 4 == 0 && Nc * R <= 4 * NT && Nc <= 4 * NT &&
                          (reinterpret_cast<uintptr_t>(replicas) & 15) == 0 && (!weight || (reinterpret_cast<uintptr_t>(weight) & 15) == 0);
    const bool e2c_regs = N % 4 == 0 && N <= 8 * NT && (reinterpret_cast<uintptr_t>(e2c) & 15) == 0;
    if (tab_regs && lds + tab_bytes <= budget) { stage_tab = 1; lds += tab_bytes; }
    if (e2c_regs && lds + e2c_bytes <= budget) { stage_e2c = 1; lds += e2c_bytes; }
    const int sel_off = (int)(lds / 4);
    lds += (size_t)k * 4;
    if (lds > budget) return SWARM_OK;
    lds = (lds + 15) / 16 * 16;
    if (lds + (size_t)cap * 8 <= budget) { a.split_off = (int)(lds / 4); lds += (size_t)cap * 8; }
    const dim3 grid((unsigned)H), block(NT);
    hipStream_t st = ctx->stream;
    if (sliced) {
        int M = 0, stride = 0;
        int32_t* cand = nullptr;
        const swarm_status rc = launch_select_slices(ctx, scores, H, N, k, &M, &stride, &cand);
        if (rc != SWARM_OK) return rc;
#define SWARM_MERGEMAP(IPT) hipLaunchKernelGGL((select_map_kernel<IPT, true>), grid, block, lds, st, scores, N, k, out_idx, a, stage_e2c, stage_tab, sel_off, cand, stride, M)
        if (M <= 4 * NT) SWARM_MERGEMAP(4);
        else if (M <= 8 * NT) SWARM_MERGEMAP(8);
        else if (M <= 16 * NT) SWARM_MERGEMAP(16);
        else if (M <= 32 * NT) SWARM_MERGEMAP(32);
        else SWARM_MERGEMAP(64);
#undef SWARM_MERGEMAP
        *launched = hipGetLastError() == hipSuccess;      // a refused launch (e.g. its LDS request) leaves the two-kernel route to the caller
        return SWARM_OK;
    }
#define SWARM_SELMAP(IPT) hipLaunchKernelGGL((select_map_kernel<IPT, false>), grid, block, lds, st, scores, N, k, out_idx, a, stage_e2c, stage_tab, sel_off, nullptr, 0, 0)
    if (NT == 256) hipLaunchKernelGGL((select_map_kernel<4, false, 256>), grid, block, lds, st, scores, N, k, out_idx, a, stage_e2c, stage_tab, sel_off, nullptr, 0, 0);
    else if (NT == 512) hipLaunchKernelGGL((select_map_kernel<4, false, 512>), grid, block, lds, st, scores, N, k, out_idx, a, stage_e2c, stage_tab, sel_off, nullptr, 0, 0);
    else if (N <= 4 * NT) SWARM_SELMAP(4);
    else if (N <= 8 * NT) SWARM_SELMAP(8);
    else if (N <= 16 * NT) SWARM_SELMAP(16);
    else if (N <= 32 * NT) SWARM_SELMAP(32);
    else SWARM_SELMAP(64);
#undef SWARM_SELMAP
    *launched = hipGetLastError() == hipSuccess;          // a refused launch leaves the two-kernel route to the caller
    return SWARM_OK;
}
