// Request mapping (Section 6.1): merge the clusters activated by a group of selections, drop the
// DRAM-resident ones, and fill one bucket per SSD by sending each cluster -- in ascending
// (replication factor, cluster id) -- to its least-loaded replica.
//
// One wavefront per group.  The merge is an LDS bitmap (atomic-or per selected entry), compacted
// in ascending cluster id.  The greedy assignment is an inherently sequential chain over the
// distinct clusters; each link is a wave-level argmin: lane d holds bucket d's load, candidate
// lanes compete with (load, lane) packed in one word and a DPP min-reduction picks the winner.
#include "common.h"

namespace {

constexpr uint32_t INF32 = 0xffffffffu;

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_min(uint32_t v) {
    const uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xF, 0xF, false);
    return min(v, o);
}

// Minimum over the first 2^STEPS lanes (valid in every one of them); other lanes hold INF32.
template <int STEPS>
__device__ __forceinline__ uint32_t low_lanes_min(uint32_t v) {
    v = dpp_min<0xB1>(v);                       // quad_perm [1,0,3,2]
    v = dpp_min<0x4E>(v);                       // quad_perm [2,3,0,1]
    if (STEPS >= 3) v = dpp_min<0x141>(v);      // row_half_mirror
    if (STEPS >= 4) v = dpp_min<0x140>(v);      // row_mirror
    if (STEPS >= 5) v = min(v, (uint32_t)__shfl_xor((int)v, 16, 64));
    if (STEPS >= 6) v = min(v, (uint32_t)__shfl_xor((int)v, 32, 64));
    return v;
}

__device__ __forceinline__ uint32_t wave_excl_scan(uint32_t v, int lane, uint32_t* total) {
    uint32_t incl = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t o = __shfl_up(incl, off, 64);
        if (lane >= off) incl += o;
    }
    *total = __shfl(incl, 63, 64);
    return incl - v;
}

struct MapArgs {
    const int32_t* sel; int S; int H; int N; const int32_t* e2c; int Nc; const int32_t* replicas; int R; int D;
    const int32_t* weight; const uint32_t* resident; int32_t* q_off; int32_t* q_cluster; int32_t* q_load; int cap;
    uint32_t* dev_flags;
};

// The greedy chain.  PACKED: bucket loads stay below 2^26, so (load << 6 | lane) fits one word and
// a single min-reduction yields the least-loaded candidate with ties to the lower SSD id.
template <int STEPS, bool PACKED>
__device__ __forceinline__ void greedy_chain(int m, int lane, const uint32_t* order, const uint32_t* mask_lo,
                                             const uint32_t* mask_hi, const uint32_t* wgt, uint32_t* assign,
                                             uint32_t& load, uint32_t& cnt) {
    for (int it = 0; it < m; ++it) {
        const uint32_t i = order[it];
        const uint64_t mask = ((uint64_t)mask_hi[i] << 32) | mask_lo[i];
        if (mask == 0) { if (lane == 0) assign[i] = INF32; continue; }
        const bool cand = (mask >> lane) & 1ull;
        int winner;
        if (PACKED) {
            const uint32_t key = cand ? ((load << 6) | (uint32_t)lane) : INF32;
            winner = (int)(low_lanes_min<STEPS>(key) & 63u);
            winner = __builtin_amdgcn_readfirstlane(winner);
        } else {
            const uint32_t key = cand ? load : INF32;
            const uint32_t best = low_lanes_min<STEPS>(key);
            const uint64_t tie = __ballot(cand && key == __builtin_amdgcn_readfirstlane((int)best));
            winner = __ffsll((unsigned long long)tie) - 1;
        }
        if (lane == winner) {
            assign[i] = ((uint32_t)winner << 24) | cnt;
            load += wgt[i];
            ++cnt;
        }
    }
}

__global__ __launch_bounds__(64) void map_requests_kernel(MapArgs a) {
    extern __shared__ uint32_t smem[];
    const int nwords = (a.Nc + 31) / 32;
    uint32_t* bitmap = smem;
    uint32_t* list = bitmap + nwords;
    uint32_t* mask_lo = list + a.cap;
    uint32_t* mask_hi = mask_lo + a.cap;
    uint32_t* wgt = mask_hi + a.cap;
    uint32_t* order = wgt + a.cap;
    uint32_t* assign = order + a.cap;
    uint32_t* off = assign + a.cap;                 // 64 words

    const int lane = threadIdx.x;
    const int64_t g = blockIdx.x;
    const int h = (int)(g % a.H);
    uint32_t flags = 0;

    for (int w = lane; w < nwords; w += 64) bitmap[w] = 0;
    __syncthreads();

    // merge: one bit per activated, non-resident cluster
    const int32_t* sel = a.sel + g * a.S;
    const int32_t* e2c = a.e2c + (size_t)h * a.N;
    for (int s = lane; s < a.S; s += 64) {
        const int32_t e = sel[s];
        if (e < 0 || e >= a.N) { flags |= SWARM_DEV_BAD_ENTRY; continue; }
        const int32_t c = e2c[e];
        if (c < 0 || c >= a.Nc) { flags |= SWARM_DEV_BAD_CLUSTER; continue; }
        if (a.resident) {
            const int64_t gc = (int64_t)h * a.Nc + c;
            if ((a.resident[gc >> 5] >> (gc & 31)) & 1u) continue;
        }
        atomicOr(&bitmap[c >> 5], 1u << (c & 31));
    }
    __syncthreads();

    // compaction in ascending cluster id
    uint32_t m = 0;
    for (int w0 = 0; w0 < nwords; w0 += 64) {
        const int w = w0 + lane;
        uint32_t bits = (w < nwords) ? bitmap[w] : 0u;
        uint32_t total;
        uint32_t pos = m + wave_excl_scan(__popc(bits), lane, &total);
        while (bits) {
            const int bit = __ffs(bits) - 1;
            bits &= bits - 1;
            if (pos < (uint32_t)a.cap) list[pos] = (uint32_t)(w * 32 + bit);
            ++pos;
        }
        m += total;
    }
    if (m > (uint32_t)a.cap) { flags |= SWARM_DEV_CAP; m = a.cap; }
    __syncthreads();

    // per item: candidate SSD mask, weight, replication factor
    const int64_t cbase = (int64_t)h * a.Nc;
    uint32_t rf_min = INF32, rf_max = 0, wsum = 0;
    for (uint32_t i = lane; i < m; i += 64) {
        const int64_t gc = cbase + list[i];
        uint64_t mask = 0;
        for (int r = 0; r < a.R; ++r) {
            const int32_t dsk = a.replicas[gc * a.R + r];
            if (dsk >= a.D) flags |= SWARM_DEV_BAD_SSD;
            else if (dsk >= 0) mask |= 1ull << dsk;
        }
        if (mask == 0) flags |= SWARM_DEV_BAD_SSD;
        mask_lo[i] = (uint32_t)mask;
        mask_hi[i] = (uint32_t)(mask >> 32);
        const uint32_t wv = a.weight ? (uint32_t)max(a.weight[gc], 0) : 1u;
        wgt[i] = wv;
        wsum += min(wv, 1u << 26);
        const uint32_t rf = __popcll(mask);
        order[i] = rf;                               // replication factor for now
        rf_min = min(rf_min, rf);
        rf_max = max(rf_max, rf);
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        rf_min = min(rf_min, (uint32_t)__shfl_xor((int)rf_min, o, 64));
        rf_max = max(rf_max, (uint32_t)__shfl_xor((int)rf_max, o, 64));
        const uint32_t ws = (uint32_t)__shfl_xor((int)wsum, o, 64);
        wsum = (wsum + ws > (1u << 26)) ? (1u << 26) : wsum + ws;
    }
    __syncthreads();

    // visiting order: stable by replication factor (identity when all factors agree)
    if (m > 0 && rf_min == rf_max) {
        for (uint32_t i = lane; i < m; i += 64) order[i] = i;
    } else if (m > 0) {
        uint32_t* rfv = assign;                      // assign is free until the chain runs
        for (uint32_t i = lane; i < m; i += 64) rfv[i] = order[i];
        __syncthreads();
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
    }
    __syncthreads();

    // greedy least-loaded assignment
    uint32_t load = 0, cnt = 0;
    const bool packed = wsum < (1u << 26);
    const int D = a.D;
    if (packed) {
        if (D <= 4) greedy_chain<2, true>(m, lane, order, mask_lo, mask_hi, wgt, assign, load, cnt);
        else if (D <= 8) greedy_chain<3, true>(m, lane, order, mask_lo, mask_hi, wgt, assign, load, cnt);
        else if (D <= 16) greedy_chain<4, true>(m, lane, order, mask_lo, mask_hi, wgt, assign, load, cnt);
        else greedy_chain<6, true>(m, lane, order, mask_lo, mask_hi, wgt, assign, load, cnt);
    } else {
        if (D <= 16) greedy_chain<4, false>(m, lane, order, mask_lo, mask_hi, wgt, assign, load, cnt);
        else greedy_chain<6, false>(m, lane, order, mask_lo, mask_hi, wgt, assign, load, cnt);
    }
    __syncthreads();

    // emit buckets SSD-major, insertion order inside a bucket
    uint32_t total;
    const uint32_t my_off = wave_excl_scan(lane < D ? cnt : 0u, lane, &total);
    off[lane] = my_off;
    int32_t* q_off = a.q_off + g * (D + 1);
    if (lane < D) {
        q_off[lane] = (int32_t)my_off;
        a.q_load[g * D + lane] = (int32_t)load;
    }
    if (lane == 0) q_off[D] = (int32_t)total;
    __syncthreads();
    int32_t* qc = a.q_cluster + g * a.cap;
    for (uint32_t i = lane; i < m; i += 64) {
        const uint32_t as = assign[i];
        if (as != INF32) qc[off[as >> 24] + (as & 0xffffffu)] = (int32_t)list[i];
    }
    for (uint32_t p = total + lane; p < (uint32_t)a.cap; p += 64) qc[p] = -1;

    if (flags) atomicOr(a.dev_flags, flags);
}

}  // namespace

swarm_status launch_map(swarm_ctx* ctx, const int32_t* sel, int64_t groups, int S, int H, int N, const int32_t* e2c,
                        int Nc, const int32_t* replicas, int R, int D, const int32_t* weight,
                        const uint32_t* resident, int32_t* q_off, int32_t* q_cluster, int32_t* q_load, int cap) {
    MapArgs a{sel, S, H, N, e2c, Nc, replicas, R, D, weight, resident, q_off, q_cluster, q_load, cap, ctx->dev_flags};
    const size_t lds = ((size_t)(Nc + 31) / 32 + (size_t)cap * 6 + 64) * 4;
    hipLaunchKernelGGL(map_requests_kernel, dim3((unsigned)groups), dim3(64), lds, ctx->stream, a);
    return swarm_check_launch(ctx, "map_requests_kernel");
}
