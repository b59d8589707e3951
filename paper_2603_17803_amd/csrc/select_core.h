// Block-level exact top-k selection on register-resident scores (device code, gfx950).
//
// Selection step (Section 2.3): the k highest scores of a row, equal scores won by the lower
// index, result in ascending index order.
//
// A block of 1024 threads holds the row as IPT consecutive scores per thread.  Scores are mapped
// to order-preserving 32-bit keys.  One pass bins every score *linearly in value* between the
// row's minimum and maximum into 2048 LDS counters (float subtraction, scaling and truncation are
// all monotone, so bin order agrees with score order); a scan finds the bin b* that holds the k-th
// largest score.  Bins above b* are selected outright; inside b* (a handful of scores for any
// smooth distribution) the exact threshold key T and the number of entries equal to T that still
// belong to the result are found by ranking the candidates against each other, or -- when b*
// holds more candidates than the ranking buffer, e.g. under massive ties -- by an exact 4 x 8-bit
// radix select restricted to b*.  A final ordered compaction (block prefix scan over the
// contiguous per-thread chunks) writes the indices in ascending order, which also makes the
// lowest-index tie-break deterministic.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "wave_ops.h"

namespace selcore {

using waveops::wave_incl_scan;

constexpr int NT = 1024;        // threads per selecting block (default form)
constexpr int NB = 2048;        // value bins
constexpr int CMAX = 1024;      // candidates ranked pairwise

template <int NTH = NT>
struct SmemT {
    static constexpr int NW = NTH / 64;
    uint32_t hist[NB];
    uint32_t cand[CMAX];
    uint32_t wave_a[16], wave_b[16];
    __attribute__((aligned(16))) uint32_t wave_kmax[16];
    __attribute__((aligned(16))) uint32_t wave_kmin[16];
    uint32_t cand_count, bstar, above, thr_key, thr_need;
    uint32_t digit, digit_above;
};
using Smem = SmemT<NT>;

// Monotone map fp32 -> uint32: larger float <=> larger key.  -0 maps to the key of +0; every
// NaN maps to key 0, below -inf.
__device__ __forceinline__ uint32_t order_key(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0u;
    if (u == 0x80000000u) u = 0u;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Value used for binning only: finite, and monotone in the key (NaN and -inf share the bottom).
__device__ __forceinline__ float bin_value(uint32_t key) {
    const uint32_t bits = (key & 0x80000000u) ? (key & 0x7fffffffu) : ~key;
    float v = __uint_as_float(bits);
    if (key == 0u) v = -3.0e38f;
    v = fminf(fmaxf(v, -3.0e38f), 3.0e38f);
    return v * 0.25f;                                   // keeps hi - v finite
}

__device__ __forceinline__ int bin_of(uint32_t key, float hi, float scale) {
    const float x = (hi - bin_value(key)) * scale;      // >= 0, non-increasing in the score
    return (int)fminf(x, (float)(NB - 1));
}


// Exclusive block scan of two counters at once.  The wave totals (at most 16) are scanned by every wave on its own (lane l
// reads total l % 16, four DPP steps inside the row of 16 lanes) instead of being read and conditionally added one by one.
template <int NTH>
__device__ __forceinline__ void block_excl_scan2(uint32_t a, uint32_t b, uint32_t& ea, uint32_t& eb, SmemT<NTH>& sm,
                                                 int lane, int wave) {
    constexpr int NW = NTH / 64;
    static_assert(NW >= 1 && NW <= 16, "one wave total per lane of a DPP row");
    const uint32_t ia = wave_incl_scan(a), ib = wave_incl_scan(b);
    if (lane == 63) { sm.wave_a[wave] = ia; sm.wave_b[wave] = ib; }
    __syncthreads();
    uint32_t ta = (lane & 15) < NW ? sm.wave_a[lane & 15] : 0u, tb = (lane & 15) < NW ? sm.wave_b[lane & 15] : 0u;
    ta += waveops::dpp_or_zero<0x111, 0xF>(ta);  tb += waveops::dpp_or_zero<0x111, 0xF>(tb);     // row_shr:1
    ta += waveops::dpp_or_zero<0x112, 0xF>(ta);  tb += waveops::dpp_or_zero<0x112, 0xF>(tb);     // row_shr:2
    if (NW > 4) { ta += waveops::dpp_or_zero<0x114, 0xF>(ta);  tb += waveops::dpp_or_zero<0x114, 0xF>(tb); }    // row_shr:4
    if (NW > 8) { ta += waveops::dpp_or_zero<0x118, 0xF>(ta);  tb += waveops::dpp_or_zero<0x118, 0xF>(tb); }    // row_shr:8: totals of waves 0..l
    const int prev = wave > 0 ? wave - 1 : 0;
    const uint32_t pa = (uint32_t)__builtin_amdgcn_readlane((int)ta, prev), pb = (uint32_t)__builtin_amdgcn_readlane((int)tb, prev);
    ea = ia - a + (wave > 0 ? pa : 0u);
    eb = ib - b + (wave > 0 ? pb : 0u);
}

// key[e] is the key of index tid*IPT + e; slots at or beyond N must hold key 0.
// All NTH threads of the block must call this.  out receives k ascending indices.
// index_offset is added to every emitted index (a block selecting inside a slice of a longer row).
// Short per-thread runs keep every score's bin in a register after the histogram pass (the candidate collection and
// the compaction then compare small integers); long runs recompute it, their registers hold the keys.
template <int IPT, int NTH = NT>
__device__ __forceinline__ void block_select(const uint32_t (&key)[IPT], int N, int k, int32_t* __restrict__ out,
                                             SmemT<NTH>& sm, int index_offset = 0) {
    constexpr int NW = NTH / 64;
    constexpr bool KEEP = IPT <= 32;                    // bins kept in registers
    constexpr int NBINS_KEPT = KEEP ? IPT : 1;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int base = tid * IPT;

    // Row extrema of the binning value.  bin_value is monotone in the key, so they are the binning values of the
    // largest and the smallest key: integer max / min per score (slots at or beyond N hold key 0, which cannot raise the
    // maximum and is kept out of the minimum), two conversions at the end.
    uint32_t kmax = 0u, kmin = 0xffffffffu;
#pragma unroll
    for (int e = 0; e < IPT; ++e) {
        kmax = max(kmax, key[e]);
        kmin = min(kmin, (base + e < N) ? key[e] : 0xffffffffu);
    }
    kmax = ~waveops::wave_min_u32(~kmax);
    kmin = waveops::wave_min_u32(kmin);
    if (lane == 0) { sm.wave_kmax[wave] = kmax; sm.wave_kmin[wave] = kmin; }
#pragma unroll
    for (int i = 0; i < NB / NTH; ++i) sm.hist[tid + i * NTH] = 0;
    if (tid == 0) { sm.cand_count = 0; sm.thr_key = 0; sm.thr_need = 0xffffffffu; }
    __syncthreads();
    {
        const uint4* pmax = reinterpret_cast<const uint4*>(sm.wave_kmax);
        const uint4* pmin = reinterpret_cast<const uint4*>(sm.wave_kmin);
#pragma unroll
        for (int w = 0; w < (NW + 3) / 4; ++w) {
            const uint4 a = pmax[w], b = pmin[w];
            if (4 * w + 0 < NW) { kmax = max(kmax, a.x); kmin = min(kmin, b.x); }
            if (4 * w + 1 < NW) { kmax = max(kmax, a.y); kmin = min(kmin, b.y); }
            if (4 * w + 2 < NW) { kmax = max(kmax, a.z); kmin = min(kmin, b.z); }
            if (4 * w + 3 < NW) { kmax = max(kmax, a.w); kmin = min(kmin, b.w); }
        }
    }
    // an empty row (N = 0) leaves kmax < kmin: hi < lo, and the scale below becomes 0
    const float hi = bin_value(kmax), lo = bin_value(kmin);
    const float range = hi - lo;
    const float scale = range > 0.f ? fminf((float)NB / range, 1.0e30f) : 0.f;

    // value histogram
    int bin[NBINS_KEPT];
    auto bin_at = [&](int e) __attribute__((always_inline)) { return KEEP ? bin[e] : bin_of(key[e], hi, scale); };
#pragma unroll
    for (int e = 0; e < IPT; ++e) {
        const int b = bin_of(key[e], hi, scale);
        if (KEEP) bin[e] = b;
        atomicAdd(&sm.hist[b], 1u);
    }
    __syncthreads();

    // bin b* holding the k-th largest: cumulative count from bin 0 (highest scores) first reaches k
    {
        constexpr int PER = NB / NTH;                   // consecutive bins per thread
        uint32_t hh[PER], sum = 0;
#pragma unroll
        for (int i = 0; i < PER; ++i) { hh[i] = sm.hist[PER * tid + i]; sum += hh[i]; }
        uint32_t before, unused;
        block_excl_scan2<NTH>(sum, 0u, before, unused, sm, lane, wave);
        if (before < (uint32_t)k && (uint32_t)k <= before + sum) {
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                if (before < (uint32_t)k && (uint32_t)k <= before + hh[i]) { sm.bstar = PER * tid + i; sm.above = before; }
                before += hh[i];
            }
        }
    }
    __syncthreads();
    const int bstar = (int)sm.bstar;
    const uint32_t need = (uint32_t)k - sm.above;       // entries of bin b* that belong to the result
    const uint32_t c = sm.hist[bstar];

    if (need < c) {
        if (__builtin_expect(c <= (uint32_t)CMAX, 1)) {           // the massive-tie path is laid out off the straight line
            // rank the candidates of b* against each other
#pragma unroll
            for (int e = 0; e < IPT; ++e)
                if (bin_at(e) == bstar) sm.cand[atomicAdd(&sm.cand_count, 1u)] = key[e];
            __syncthreads();
            for (uint32_t t = tid; t < c; t += NTH) {
                const uint32_t mine = sm.cand[t];
                uint32_t gt = 0, eq = 0;
                for (uint32_t j = 0; j < c; ++j) {
                    const uint32_t other = sm.cand[j];
                    gt += other > mine;
                    eq += other == mine;
                }
                if (gt < need && need <= gt + eq) { sm.thr_key = mine; sm.thr_need = need - gt; }
            }
            __syncthreads();
        } else {
            // exact radix select restricted to bin b* (hist[0..256) reused as digit counters)
            uint32_t prefix = 0, mask = 0, rem = need;
            for (int shift = 24; shift >= 0; shift -= 8) {
                __syncthreads();
                if (tid < 256) sm.hist[tid] = 0;
                __syncthreads();
#pragma unroll
                for (int e = 0; e < IPT; ++e)
                    if (bin_at(e) == bstar && (key[e] & mask) == prefix)
                        atomicAdd(&sm.hist[(key[e] >> shift) & 255u], 1u);
                __syncthreads();
                if (wave == 0) {
                    const uint32_t h0 = sm.hist[4 * lane], h1 = sm.hist[4 * lane + 1], h2 = sm.hist[4 * lane + 2],
                                   h3 = sm.hist[4 * lane + 3];
                    const uint32_t tot = h0 + h1 + h2 + h3;
                    uint32_t incl = tot;
#pragma unroll
                    for (int off = 1; off < 64; off <<= 1) {
                        const uint32_t v = __shfl_down(incl, off, 64);
                        if (lane + off < 64) incl += v;
                    }
                    uint32_t above = incl - tot;
                    const uint32_t hh[4] = {h0, h1, h2, h3};
#pragma unroll
                    for (int j = 3; j >= 0; --j) {
                        if (above < rem && rem <= above + hh[j]) { sm.digit = 4 * lane + j; sm.digit_above = above; }
                        above += hh[j];
                    }
                }
                __syncthreads();
                prefix |= sm.digit << shift;
                mask |= 0xffu << shift;
                rem -= sm.digit_above;
            }
            __syncthreads();
            if (tid == 0) { sm.thr_key = prefix; sm.thr_need = rem; }
            __syncthreads();
        }
    }
    const uint32_t T = sm.thr_key, need_eq = sm.thr_need;   // need == c: T = 0, every candidate is taken

    // ordered compaction.  A score is taken outright when it lies in a bin above b*, or in b* above the threshold key;
    // scores equal to the threshold key are taken in index order until need_eq of them are in.
    uint32_t gt = 0, eq = 0;
    uint32_t take_mask = 0, eq_mask = 0;                // bit e (KEEP only; IPT <= 32)
#pragma unroll
    for (int e = 0; e < IPT; ++e) {
        const int b = bin_at(e);
        const bool g = (b < bstar) || (b == bstar && key[e] > T);
        const bool q = (b == bstar && key[e] == T);
        gt += g;
        eq += q;
        if (KEEP) { take_mask |= (uint32_t)g << e; eq_mask |= (uint32_t)q << e; }
    }
    uint32_t gt_before, eq_before;
    block_excl_scan2<NTH>(gt, eq, gt_before, eq_before, sm, lane, wave);
    uint32_t pos = gt_before + min(eq_before, need_eq);
    if (KEEP) {
        // the equal scores this thread still takes: its first (need_eq - eq_before) of them
        const uint32_t room = need_eq > eq_before ? need_eq - eq_before : 0u;
        uint32_t m = eq_mask;
        for (uint32_t i = 0; i < room && m; ++i) { take_mask |= m & (0u - m); m &= m - 1u; }
        while (take_mask) {
            const int e = __ffs(take_mask) - 1;
            take_mask &= take_mask - 1u;
            if (pos < (uint32_t)k) out[pos] = index_offset + base + e;     // pos < k always holds; the guard keeps a slip in bounds
            ++pos;
        }
    } else {
        uint32_t eq_seen = eq_before;
#pragma unroll
        for (int e = 0; e < IPT; ++e) {
            const int b = bin_of(key[e], hi, scale);
            const bool is_eq = (b == bstar && key[e] == T);
            const bool take = (b < bstar) || (b == bstar && key[e] > T) || (is_eq && eq_seen < need_eq);
            eq_seen += is_eq;
            if (take) {
                if (pos < (uint32_t)k) out[pos] = index_offset + base + e;
                ++pos;
            }
        }
    }
}

// Loads IPT consecutive scores of a row into keys (slots beyond N get key 0).
template <int IPT>
__device__ __forceinline__ void load_keys(const float* __restrict__ row, int N, uint32_t (&key)[IPT]) {
    const int base = threadIdx.x * IPT;
    if (((reinterpret_cast<uintptr_t>(row) & 15) == 0) && base + IPT <= N) {
        const float4* p = reinterpret_cast<const float4*>(row + base);
#pragma unroll
        for (int e = 0; e < IPT / 4; ++e) {
            const float4 v = p[e];
            key[4 * e] = order_key(v.x);
            key[4 * e + 1] = order_key(v.y);
            key[4 * e + 2] = order_key(v.z);
            key[4 * e + 3] = order_key(v.w);
        }
    } else {
#pragma unroll
        for (int e = 0; e < IPT; ++e) key[e] = (base + e < N) ? order_key(row[base + e]) : 0u;
    }
}

}  // namespace selcore
