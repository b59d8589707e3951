// Medoid-indexed retrieval helpers around the mapping step (Section 5.2, Tier 1, and Section 6.1):
//   cluster expansion -- the clusters activated through their medoids are merged (each once, ascending
//   id) and replaced by their member entries, the input of the entry-level mapping step;
//   submission order  -- the buckets built by the mapping step are drained head by head: batch b is the
//   b-th item of every bucket that has one, in ascending SSD id.
#include "common.h"
#include "wave_ops.h"

namespace {

using waveops::wave_excl_scan;

constexpr int EXP_THREADS = 256;

// One workgroup per group.  LDS: bitmap of activated clusters (Nc bits) + one partial sum per thread.
__global__ __launch_bounds__(EXP_THREADS) void expand_clusters_kernel(const int32_t* __restrict__ clusters, int Sc, int H, int Nc,
                                                                      const int32_t* __restrict__ cl_off,
                                                                      const int32_t* __restrict__ cl_entries, int E,
                                                                      int32_t* __restrict__ entries, int32_t* __restrict__ count,
                                                                      int cap_e, uint32_t* __restrict__ dev_flags) {
    extern __shared__ uint32_t smem[];
    const int nwords = (Nc + 31) / 32;
    uint32_t* bitmap = smem;
    uint32_t* wave_tot = smem + nwords;            // EXP_THREADS / 64 words
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t g = blockIdx.x;
    const int h = (int)(g % H);
    uint32_t flags = 0;
    for (int w = tid; w < nwords; w += EXP_THREADS) bitmap[w] = 0;
    __syncthreads();
    for (int s = tid; s < Sc; s += EXP_THREADS) {
        const int32_t c = clusters[g * Sc + s];
        if (c == -1) continue;
        if (c < 0 || c >= Nc) { flags |= SWARM_DEV_BAD_CLUSTER; continue; }
        atomicOr(&bitmap[c >> 5], 1u << (c & 31));
    }
    __syncthreads();
    // thread t owns a contiguous run of bitmap words, so that thread order is cluster order
    const int wpt = (nwords + EXP_THREADS - 1) / EXP_THREADS;
    const int w0 = min(tid * wpt, nwords), w1 = min(w0 + wpt, nwords);
    const int32_t* off = cl_off + (size_t)h * (Nc + 1);
    uint32_t mine = 0;
    for (int w = w0; w < w1; ++w) {
        uint32_t bits = bitmap[w];
        while (bits) {
            const int c = w * 32 + __ffs(bits) - 1;
            bits &= bits - 1;
            const int32_t lo = off[c], hi = off[c + 1];
            if (lo < 0 || hi < lo || hi > E) { flags |= SWARM_DEV_BAD_CLUSTER; continue; }
            mine += (uint32_t)(hi - lo);
        }
    }
    uint32_t wtot;
    uint32_t pos = wave_excl_scan(mine, &wtot);
    if (lane == 0) wave_tot[wave] = wtot;
    __syncthreads();
    uint32_t total = 0;
    for (int w = 0; w < EXP_THREADS / 64; ++w) {
        if (w < wave) pos += wave_tot[w];
        total += wave_tot[w];
    }
    const int32_t* ent = cl_entries + (size_t)h * E;
    int32_t* out = entries + g * cap_e;
    for (int w = w0; w < w1; ++w) {
        uint32_t bits = bitmap[w];
        while (bits) {
            const int c = w * 32 + __ffs(bits) - 1;
            bits &= bits - 1;
            const int32_t lo = off[c], hi = off[c + 1];
            if (lo < 0 || hi < lo || hi > E) continue;
            for (int32_t p = lo; p < hi; ++p, ++pos)
                if (pos < (uint32_t)cap_e) out[pos] = ent[p];
        }
    }
    if (total > (uint32_t)cap_e) { flags |= SWARM_DEV_CAP; total = cap_e; }
    if (tid == 0) count[g] = (int32_t)total;
    for (uint32_t p = total + tid; p < (uint32_t)cap_e; p += EXP_THREADS) out[p] = -1;
    if (flags) atomicOr(dev_flags, flags);
}

// One workgroup per group, one thread per routed item: the item at position pos of bucket d goes to
// rank = sum over buckets of min(length, pos) + number of lower-numbered buckets longer than pos.
__global__ __launch_bounds__(256) void submission_order_kernel(const int32_t* __restrict__ q_off, const int32_t* __restrict__ q_cluster,
                                                               int D, int cap, int32_t* __restrict__ order,
                                                               int32_t* __restrict__ batch_off, int32_t* __restrict__ nb,
                                                               uint32_t* __restrict__ dev_flags) {
    __shared__ int32_t off[65];
    const int64_t g = blockIdx.x;
    for (int d = threadIdx.x; d <= D; d += 256) off[d] = q_off[g * (D + 1) + d];
    __syncthreads();
    // offsets that are not a non-decreasing sequence from 0 to at most cap would send ranks out of range:
    // such a group gets an empty order and a flag (every thread takes the same decision)
    bool bad = off[0] != 0 || off[D] > cap;
    for (int e = 0; e < D; ++e) bad |= off[e + 1] < off[e];
    if (bad) {
        for (int32_t p = threadIdx.x; p < cap; p += 256) order[g * cap + p] = -1;
        for (int32_t b = threadIdx.x; b <= cap; b += 256) batch_off[g * (cap + 1) + b] = 0;
        if (threadIdx.x == 0) { nb[g] = 0; atomicOr(dev_flags, SWARM_DEV_BAD_OFFSETS); }
        return;
    }
    const int32_t total = off[D];
    for (int32_t p = threadIdx.x; p < cap; p += 256) {
        if (p >= total) { order[g * cap + p] = -1; continue; }
        int d = 0;
        while (d + 1 < D && off[d + 1] <= p) ++d;
        const int32_t pos = p - off[d];
        int32_t rank = 0;
        for (int e = 0; e < D; ++e) {
            const int32_t len = off[e + 1] - off[e];
            rank += min(len, pos) + ((e < d && len > pos) ? 1 : 0);
        }
        order[g * cap + rank] = q_cluster[g * cap + p];
    }
    int32_t longest = 0;
    for (int e = 0; e < D; ++e) longest = max(longest, off[e + 1] - off[e]);
    for (int32_t b = threadIdx.x; b <= cap; b += 256) {
        int32_t start = 0;
        for (int e = 0; e < D; ++e) start += min(off[e + 1] - off[e], b);
        batch_off[g * (cap + 1) + b] = min(start, total);
    }
    if (threadIdx.x == 0) nb[g] = longest;
}

}  // namespace

swarm_status launch_expand_clusters(swarm_ctx* ctx, const int32_t* clusters, int64_t groups, int Sc, int H, int Nc,
                                    const int32_t* cl_off, const int32_t* cl_entries, int E, int32_t* entries, int32_t* count,
                                    int cap_e) {
    const size_t lds = ((size_t)(Nc + 31) / 32 + EXP_THREADS / 64) * 4;
    hipLaunchKernelGGL(expand_clusters_kernel, dim3((unsigned)groups), dim3(EXP_THREADS), lds, ctx->stream, clusters, Sc, H, Nc,
                       cl_off, cl_entries, E, entries, count, cap_e, ctx->dev_flags);
    return swarm_check_launch(ctx, "expand_clusters_kernel");
}

swarm_status launch_submission_order(swarm_ctx* ctx, const int32_t* q_off, const int32_t* q_cluster, int64_t groups, int D, int cap,
                                     int32_t* order, int32_t* batch_off, int32_t* nb) {
    hipLaunchKernelGGL(submission_order_kernel, dim3((unsigned)groups), dim3(256), 0, ctx->stream, q_off, q_cluster, D, cap, order,
                       batch_off, nb, ctx->dev_flags);
    return swarm_check_launch(ctx, "submission_order_kernel");
}
