// Co-activation density and medoid queue (Section 5.1: co-activation probability of Step 1, distance
// of Step 2, density and descending medoid queue of Algorithm 1's Step 3), one streaming pass over the
// count matrix per quantity.
//
//   total  = sum of all C[k][l];  P(i,j) = C[i][j] / total;  d(i,j) = 1 - P(i,j)   (fp64)
//   rho[i] = number of j with d(i,j) <= tau
// d is a non-increasing function of the integer count (one correctly rounded division, one
// subtraction), so "d <= tau" is "count >= c*" for a single integer c* per head.  c* is found by
// bisection with exactly the fp64 expression above; the pass over C is then an integer
// compare-and-count at memory speed, and takes the same decisions as evaluating d per element.
#include "common.h"
#include "wave_ops.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int ROWS_PER_BLOCK = 4;        // one wave per row of C

__global__ void totals_init_kernel(int64_t* __restrict__ totals, const int64_t* __restrict__ totals_in, int H) {
    const int h = blockIdx.x * blockDim.x + threadIdx.x;
    if (h < H) totals[h] = totals_in ? totals_in[h] : 0;
}

__device__ __forceinline__ int64_t wave_sum_i64(int64_t v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;                               // valid in lane 0
}

// grand total per head: every wave sums rows, the workgroup adds one partial total to the head's total
// (few atomics per address: thousands of them on eight addresses cost more than the sweep itself)
__global__ __launch_bounds__(256) void row_total_kernel(const int32_t* __restrict__ C, int N, int64_t* __restrict__ totals) {
    __shared__ int64_t part[ROWS_PER_BLOCK];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int h = blockIdx.y;
    int64_t s = 0;
    for (int row = blockIdx.x * ROWS_PER_BLOCK + wave; row < N; row += gridDim.x * ROWS_PER_BLOCK) {
        const int32_t* r = C + ((size_t)h * N + row) * N;
        if ((N & 3) == 0) {
            const v4i* r4 = reinterpret_cast<const v4i*>(r);
            for (int i = lane; i < N / 4; i += 64) {
                const v4i v = __builtin_nontemporal_load(r4 + i);
                s += (int64_t)v.x + v.y + v.z + v.w;
            }
        } else {
            for (int i = lane; i < N; i += 64) s += r[i];
        }
    }
    s = wave_sum_i64(s);
    if (lane == 0) part[wave] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        int64_t t = 0;
#pragma unroll
        for (int w = 0; w < ROWS_PER_BLOCK; ++w) t += part[w];
        atomicAdd(reinterpret_cast<unsigned long long*>(totals + h), (unsigned long long)t);
    }
}

// smallest count c in [0, 2^31) whose distance passes the radius test; 2^31 when none does
__device__ __forceinline__ int64_t count_threshold(int64_t total, double tau, bool strict) {
    if (total == 0) return (int64_t)1 << 31;             // P undefined: no pair counts
    const double t = (double)total;
    auto pass = [&](int64_t c) {
        const double d = 1.0 - (double)c / t;
        return strict ? d < tau : d <= tau;
    };
    if (!pass(((int64_t)1 << 31) - 1)) return (int64_t)1 << 31;
    int64_t lo = 0, hi = ((int64_t)1 << 31) - 1;          // pass(hi) holds
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (pass(mid)) hi = mid; else lo = mid + 1;
    }
    return lo;
}

__global__ __launch_bounds__(256) void density_count_kernel(const int32_t* __restrict__ C, int N, const int64_t* __restrict__ totals,
                                                            double tau, uint32_t flags, int32_t* __restrict__ rho) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int h = blockIdx.y;
    const int row = blockIdx.x * ROWS_PER_BLOCK + wave;
    if (row >= N) return;
    const int64_t cstar = count_threshold(totals[h], tau, flags & SWARM_RHO_STRICT);
    const int32_t* r = C + ((size_t)h * N + row) * N;
    int32_t count = 0;
    if (cstar <= 0x7fffffffll) {
        const int32_t c32 = (int32_t)cstar;
        if ((N & 3) == 0) {
            const v4i* r4 = reinterpret_cast<const v4i*>(r);
            for (int i = lane; i < N / 4; i += 64) {
                const v4i v = __builtin_nontemporal_load(r4 + i);
                count += (v.x >= c32) + (v.y >= c32) + (v.z >= c32) + (v.w >= c32);
            }
        } else {
            for (int i = lane; i < N; i += 64) count += r[i] >= c32;
        }
        if ((flags & SWARM_RHO_EXCLUDE_SELF) && lane == 0) count -= r[row] >= c32;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) count += __shfl_down(count, off, 64);
    if (lane == 0) rho[(size_t)h * N + row] = count;
}

// Grand total of A^T A per head straight from the trace, and the threshold that goes with it, for a
// build that counts the density in its own epilogue: total = sum over trace rows of the square of the
// row's number of activated entries (each of a row's activated pairs adds one to C).
__global__ __launch_bounds__(256) void trace_total_threshold_kernel(const int32_t* __restrict__ row_count, int nrows, double tau,
                                                                    uint32_t flags, int64_t* __restrict__ totals,
                                                                    int64_t* __restrict__ cstar) {
    __shared__ int64_t part[4];
    const int h = blockIdx.x;
    int64_t sum = 0;
    for (int r = threadIdx.x; r < nrows; r += 256) {
        const int64_t n = row_count[(size_t)h * nrows + r];
        sum += n * n;
    }
    sum = wave_sum_i64(sum);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        const int64_t total = part[0] + part[1] + part[2] + part[3];
        totals[h] = total;
        cstar[h] = count_threshold(total, tau, flags & SWARM_RHO_STRICT);
    }
}

// j = i left out of the density: one less where the diagonal element itself reaches the threshold
__global__ void rho_exclude_self_kernel(const int32_t* __restrict__ C, int N, const int64_t* __restrict__ cstar, int32_t* __restrict__ rho) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x, h = blockIdx.y;
    if (i >= N) return;
    if ((int64_t)C[((size_t)h * N + i) * N + i] >= cstar[h]) rho[(size_t)h * N + i] -= 1;
}

// Position of entry i in the medoid queue = entries with a higher density + entries with the same
// density and a lower id: N^2 comparisons per head, tiled through LDS.  A workgroup ranks 256 entries;
// its four quarters (256 threads each) take a quarter of every staged tile of 1024 densities, and the
// partial ranks meet in LDS: four times the waves per compute unit of one thread per entry.
constexpr int RANK_ENTRIES = 256, RANK_PARTS = 4, RANK_TILE = 1024;

__global__ __launch_bounds__(RANK_ENTRIES * RANK_PARTS) void medoid_rank_kernel(const int32_t* __restrict__ rho, int N,
                                                                                  int32_t* __restrict__ queue) {
    __shared__ int32_t tile[RANK_TILE];
    __shared__ int32_t partial[RANK_PARTS - 1][RANK_ENTRIES];
    const int h = blockIdx.y;
    const int32_t* rh = rho + (size_t)h * N;
    const int e = threadIdx.x % RANK_ENTRIES, part = threadIdx.x / RANK_ENTRIES;
    const int i = blockIdx.x * RANK_ENTRIES + e;
    const int32_t mine = i < N ? rh[i] : 0;
    constexpr int SUB = RANK_TILE / RANK_PARTS;
    int32_t rank = 0;
    for (int j0 = 0; j0 < N; j0 += RANK_TILE) {
        __syncthreads();
        tile[threadIdx.x] = (j0 + (int)threadIdx.x < N) ? rh[j0 + threadIdx.x] : -1;
        __syncthreads();
        // this quarter's slice [s0, s0 + lim) of the tile; entries below i win ties, entries above lose them:
        // count (rho_j >= mine) for j < i and (rho_j > mine) for j > i, split at j = i
        const int s0 = part * SUB;
        const int lim = max(0, min(SUB, N - j0 - s0));
        const int below = max(0, min(lim, i - j0 - s0));
        const int32_t* t = tile + s0;
#pragma unroll 8
        for (int u = 0; u < below; ++u) rank += t[u] >= mine;
#pragma unroll 8
        for (int u = below; u < lim; ++u) rank += t[u] > mine;
    }
    if (part > 0) partial[part - 1][e] = rank;
    __syncthreads();
    if (part == 0 && i < N) {
#pragma unroll
        for (int p = 0; p < RANK_PARTS - 1; ++p) rank += partial[p][e];
        queue[(size_t)h * N + rank] = i;
    }
}

}  // namespace

swarm_status launch_density(swarm_ctx* ctx, const int32_t* C, int H, int N, const int64_t* totals_in, double tau,
                            uint32_t flags, int32_t* rho, int32_t* queue, int64_t* totals) {
    hipLaunchKernelGGL(totals_init_kernel, dim3((unsigned)((H + 63) / 64)), dim3(64), 0, ctx->stream, totals, totals_in, H);
    swarm_status st = swarm_check_launch(ctx, "totals_init_kernel");
    if (st != SWARM_OK) return st;
    const dim3 grid((unsigned)((N + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK), (unsigned)H);
    if (!totals_in) {
        const unsigned per_head = grid.x < 512u ? grid.x : 512u;
        hipLaunchKernelGGL(row_total_kernel, dim3(per_head, (unsigned)H), dim3(256), 0, ctx->stream, C, N, totals);
        st = swarm_check_launch(ctx, "row_total_kernel");
        if (st != SWARM_OK) return st;
    }
    hipLaunchKernelGGL(density_count_kernel, grid, dim3(256), 0, ctx->stream, C, N, totals, tau, flags, rho);
    st = swarm_check_launch(ctx, "density_count_kernel");
    if (st != SWARM_OK || !queue) return st;
    return launch_medoid_rank(ctx, rho, H, N, queue);
}

swarm_status launch_medoid_rank(swarm_ctx* ctx, const int32_t* rho, int H, int N, int32_t* queue) {
    hipLaunchKernelGGL(medoid_rank_kernel, dim3((unsigned)((N + RANK_ENTRIES - 1) / RANK_ENTRIES), (unsigned)H),
                       dim3(RANK_ENTRIES * RANK_PARTS), 0, ctx->stream, rho, N, queue);
    return swarm_check_launch(ctx, "medoid_rank_kernel");
}

swarm_status launch_trace_totals_thresholds(swarm_ctx* ctx, const int32_t* row_count, int H, int nrows, double tau, uint32_t flags,
                                            int64_t* totals, int64_t* cstar) {
    hipLaunchKernelGGL(trace_total_threshold_kernel, dim3((unsigned)H), dim3(256), 0, ctx->stream, row_count, nrows, tau, flags,
                       totals, cstar);
    return swarm_check_launch(ctx, "trace_total_threshold_kernel");
}

swarm_status launch_rho_exclude_self(swarm_ctx* ctx, const int32_t* C, int H, int N, const int64_t* cstar, int32_t* rho) {
    hipLaunchKernelGGL(rho_exclude_self_kernel, dim3((unsigned)((N + 255) / 256), (unsigned)H), dim3(256), 0, ctx->stream, C, N, cstar,
                       rho);
    return swarm_check_launch(ctx, "rho_exclude_self_kernel");
}
