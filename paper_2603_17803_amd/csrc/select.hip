// Selection step (Section 2.3) as a stand-alone kernel: one 1024-thread block per score row.
//
// Rows of up to 65536 scores are held in registers and selected by selcore::block_select (value
// binning + exact refinement, see select_core.h).  Longer rows use the streaming kernel below: an
// exact radix select that re-reads the row from memory for each of its four 8-bit digit passes.
#include "common.h"
#include "select_core.h"

namespace {

using selcore::order_key;

template <int IPT, int NTH = selcore::NT>
__global__ __launch_bounds__(NTH) void topk_select_kernel(const float* __restrict__ scores, int N, int k,
                                                           int32_t* __restrict__ out_idx) {
    __shared__ selcore::SmemT<NTH> sm;
    uint32_t key[IPT];
    selcore::load_keys<IPT>(scores + (size_t)blockIdx.x * N, N, key);
    selcore::block_select<IPT, NTH>(key, N, k, out_idx + (size_t)blockIdx.x * k, sm);
}

// ---- long rows, few of them: two stages -----------------------------------------------------------
// A single workgroup selecting a 65536-entry row spends tens of microseconds on it.  When there are too
// few rows to fill the device, a row is cut into slices of SLICE entries: every slice keeps its own
// top-min(k, slice length) (exactly, with the same tie-break), and one workgroup per row then selects
// among the slices' winners.  An entry dropped by its slice is beaten by that many entries of the same
// slice, each with a higher score or an equal score and a lower index, so it cannot belong to the
// row's result; the winners are listed in ascending entry id, so position order is index order and
// the lowest-index tie-break carries over.
constexpr int SLICE = 8192, SLICE_IPT = 8;

__global__ __launch_bounds__(selcore::NT) void topk_slice_kernel(const float* __restrict__ scores, int N, int k,
                                                                 int32_t* __restrict__ cand, int cand_stride) {
    __shared__ selcore::Smem sm;
    const int p = blockIdx.x;
    const int64_t row = blockIdx.y;
    const int lo = p * SLICE, len = min(SLICE, N - lo);
    const int kk = min(k, len);
    uint32_t key[SLICE_IPT];
    selcore::load_keys<SLICE_IPT>(scores + row * N + lo, len, key);
    // slices before this one are full, so their winner counts are min(k, SLICE) each
    selcore::block_select<SLICE_IPT>(key, len, kk, cand + row * cand_stride + (size_t)p * min(k, SLICE), sm, lo);
}

template <int IPT>
__global__ __launch_bounds__(selcore::NT) void topk_merge_kernel(const float* __restrict__ scores, int N, int k,
                                                                 const int32_t* __restrict__ cand, int cand_stride, int M,
                                                                 int32_t* __restrict__ out_idx) {
    __shared__ selcore::Smem sm;
    const int64_t row = blockIdx.x;
    const int32_t* c = cand + row * cand_stride;
    const float* s = scores + row * N;
    uint32_t key[IPT];
    const int base = threadIdx.x * IPT;
#pragma unroll
    for (int e = 0; e < IPT; ++e) key[e] = (base + e < M) ? order_key(s[c[base + e]]) : 0u;
    int32_t* out = out_idx + row * k;
    selcore::block_select<IPT>(key, M, k, out, sm);      // positions in the winners' list, ascending
    __syncthreads();
    for (int j = threadIdx.x; j < k; j += selcore::NT) out[j] = c[out[j]];
}

constexpr int SEL_THREADS = 1024;

// Streaming fallback for rows longer than 65536 entries.
__global__ __launch_bounds__(SEL_THREADS) void topk_select_stream_kernel(const float* __restrict__ scores, int N, int k,
                                                                         int32_t* __restrict__ out_idx) {
    __shared__ uint32_t hist[256];
    __shared__ uint32_t s_digit, s_above;
    __shared__ uint32_t wave_gt[SEL_THREADS / 64], wave_eq[SEL_THREADS / 64];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float* s = scores + (size_t)blockIdx.x * N;
    int32_t* out = out_idx + (size_t)blockIdx.x * k;

    uint32_t prefix = 0, mask = 0, need = (uint32_t)k;
    for (int shift = 24; shift >= 0; shift -= 8) {
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        for (int i = tid; i < N; i += SEL_THREADS) {
            const uint32_t key = order_key(s[i]);
            if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
        }
        __syncthreads();
        if (wave == 0) {
            // lane l owns digits 4l..4l+3; find the digit whose suffix count first reaches `need`
            const uint32_t h0 = hist[4 * lane], h1 = hist[4 * lane + 1], h2 = hist[4 * lane + 2], h3 = hist[4 * lane + 3];
            const uint32_t tot = h0 + h1 + h2 + h3;
            uint32_t incl = tot;                                  // inclusive suffix sum over lanes >= l
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const uint32_t v = __shfl_down(incl, off, 64);
                if (lane + off < 64) incl += v;
            }
            uint32_t above = incl - tot;                          // entries in digits of higher lanes
            const uint32_t hh[4] = {h0, h1, h2, h3};
#pragma unroll
            for (int j = 3; j >= 0; --j) {
                if (above < need && need <= above + hh[j]) { s_digit = 4 * lane + j; s_above = above; }
                above += hh[j];
            }
        }
        __syncthreads();
        prefix |= s_digit << shift;
        mask |= 0xffu << shift;
        need -= s_above;
        __syncthreads();
    }
    const uint32_t T = prefix;

    // ordered compaction: thread t owns the contiguous chunk [t*chunk, (t+1)*chunk)
    const int chunk = (N + SEL_THREADS - 1) / SEL_THREADS;
    const int lo = min(tid * chunk, N), hi = min(lo + chunk, N);
    uint32_t gt = 0, eq = 0;
    for (int i = lo; i < hi; ++i) {
        const uint32_t key = order_key(s[i]);
        gt += key > T;
        eq += key == T;
    }
    uint32_t gt_incl = gt, eq_incl = eq;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t a = __shfl_up(gt_incl, off, 64), b = __shfl_up(eq_incl, off, 64);
        if (lane >= off) { gt_incl += a; eq_incl += b; }
    }
    if (lane == 63) { wave_gt[wave] = gt_incl; wave_eq[wave] = eq_incl; }
    __syncthreads();
    uint32_t gt_before = gt_incl - gt, eq_before = eq_incl - eq;
    for (int w = 0; w < wave; ++w) { gt_before += wave_gt[w]; eq_before += wave_eq[w]; }

    uint32_t pos = gt_before + min(eq_before, need);
    uint32_t eq_seen = eq_before;
    for (int i = lo; i < hi; ++i) {
        const uint32_t key = order_key(s[i]);
        const bool take = key > T || (key == T && eq_seen < need);
        eq_seen += key == T;
        if (take) {
            if (pos < (uint32_t)k) out[pos] = i;      // pos < k always holds; the guard keeps a logic slip in bounds
            ++pos;
        }
    }
}

}  // namespace

bool select_uses_slices(int64_t rows, int N, int k) {
    if (N <= 2 * SLICE || rows > 32) return false;
    const int64_t P = (N + SLICE - 1) / SLICE;
    const int64_t M = (P - 1) * (k < SLICE ? k : SLICE) + (k < N - (P - 1) * SLICE ? k : N - (P - 1) * SLICE);
    return M <= N / 2 && M <= 64 * selcore::NT;
}

size_t select_cand_bytes(int64_t rows, int N, int k) {
    if (!select_uses_slices(rows, N, k)) return 0;
    const int64_t P = (N + SLICE - 1) / SLICE;
    return sizeof(int32_t) * (size_t)rows * (size_t)(P * (k < SLICE ? k : SLICE));
}

// First stage of the sliced selection: the slices' winners of every row into *cand_out ([rows][*stride], *M of them per
// row), which is the context's scratch (grown on demand) or the fixed scratch when one is given.
swarm_status launch_select_slices(swarm_ctx* ctx, const float* scores, int64_t rows, int N, int k, int* M_out, int* stride_out,
                                  int32_t** cand_out, const swarm_fixed_scratch* fixed) {
    const int P = (N + SLICE - 1) / SLICE;
    const int per = k < SLICE ? k : SLICE;
    const int last = N - (P - 1) * SLICE;
    *M_out = (P - 1) * per + (k < last ? k : last);
    *stride_out = P * per;
    const size_t need = sizeof(int32_t) * (size_t)rows * *stride_out;
    int32_t* cand = nullptr;
    if (fixed) {
        if (need > fixed->cand_bytes) {
            snprintf(ctx->err, sizeof(ctx->err), "select: the slices' winners need %zu bytes, the fixed scratch has %zu", need, fixed->cand_bytes);
            return SWARM_EINVAL;
        }
        cand = fixed->cand;
    } else {
        const swarm_status rc = swarm_grow(ctx, reinterpret_cast<void**>(&ctx->cand), &ctx->cand_bytes, need);
        if (rc != SWARM_OK) return rc;
        cand = ctx->cand;
    }
    *cand_out = cand;
    hipLaunchKernelGGL(topk_slice_kernel, dim3((unsigned)P, (unsigned)rows), dim3(selcore::NT), 0, ctx->stream, scores, N, k, cand,
                       *stride_out);
    return swarm_check_launch(ctx, "topk_slice_kernel");
}

swarm_status launch_select(swarm_ctx* ctx, const float* scores, int64_t rows, int N, int k, int32_t* out_idx,
                           const swarm_fixed_scratch* fixed) {
    const dim3 grid((unsigned)rows), block(selcore::NT);
    hipStream_t st = ctx->stream;
    if (select_uses_slices(rows, N, k)) {
        int M = 0, stride = 0;
        int32_t* cand = nullptr;
        const swarm_status rc = launch_select_slices(ctx, scores, rows, N, k, &M, &stride, &cand, fixed);
        if (rc != SWARM_OK) return rc;
        if (M <= 4 * selcore::NT) hipLaunchKernelGGL(topk_merge_kernel<4>, grid, block, 0, st, scores, N, k, cand, stride, M, out_idx);
        else if (M <= 8 * selcore::NT) hipLaunchKernelGGL(topk_merge_kernel<8>, grid, block, 0, st, scores, N, k, cand, stride, M, out_idx);
        else if (M <= 16 * selcore::NT) hipLaunchKernelGGL(topk_merge_kernel<16>, grid, block, 0, st, scores, N, k, cand, stride, M, out_idx);
        else if (M <= 32 * selcore::NT) hipLaunchKernelGGL(topk_merge_kernel<32>, grid, block, 0, st, scores, N, k, cand, stride, M, out_idx);
        else hipLaunchKernelGGL(topk_merge_kernel<64>, grid, block, 0, st, scores, N, k, cand, stride, M, out_idx);
        return swarm_check_launch(ctx, "topk_merge_kernel");
    }
    // Short rows take smaller blocks, four scores per thread: measured per row of 2048 scores, 512 threads select in
    // 3.6 us where 1024 (half of them idle, sixteen waves at every barrier) take 5.6 us; rows of 8192 are fastest with 1024.
    if (N <= 4 * 256) {
        hipLaunchKernelGGL((topk_select_kernel<4, 256>), grid, dim3(256), 0, st, scores, N, k, out_idx);
        return swarm_check_launch(ctx, "topk_select_kernel");
    }
    if (N <= 4 * 512) {
        hipLaunchKernelGGL((topk_select_kernel<4, 512>), grid, dim3(512), 0, st, scores, N, k, out_idx);
        return swarm_check_launch(ctx, "topk_select_kernel");
    }
    if (N <= 4 * selcore::NT) hipLaunchKernelGGL(topk_select_kernel<4>, grid, block, 0, st, scores, N, k, out_idx);
    else if (N <= 8 * selcore::NT) hipLaunchKernelGGL(topk_select_kernel<8>, grid, block, 0, st, scores, N, k, out_idx);
    else if (N <= 16 * selcore::NT) hipLaunchKernelGGL(topk_select_kernel<16>, grid, block, 0, st, scores, N, k, out_idx);
    else if (N <= 32 * selcore::NT) hipLaunchKernelGGL(topk_select_kernel<32>, grid, block, 0, st, scores, N, k, out_idx);
    else if (N <= 64 * selcore::NT) hipLaunchKernelGGL(topk_select_kernel<64>, grid, block, 0, st, scores, N, k, out_idx);
    else hipLaunchKernelGGL(topk_select_stream_kernel, grid, block, 0, st, scores, N, k, out_idx);
    return swarm_check_launch(ctx, "topk_select_kernel");
}
