// Cluster maintenance over the local window (Section 6.2): for every newly generated entry e and every
// cluster medoid m_i, f(e, m_i) = number of the window's W steps in which both are activated,
// d = 1 - f / W (fp64), and e joins every cluster with d < tau; a joining entry goes to the cluster's
// next SSD, (id_i + |C_i| + 1) mod D, with |C_i| growing as entries join in the order given.
//
// f is a thin (new entries x medoids) slice of the window's A^T A.  The window's trace is built as
// bits (the same builder as for the full co-activation matrix), so a count is a handful of
// AND + popcount operations on the two entries' 16-byte words.
#include "common.h"

namespace {

typedef unsigned int v4u __attribute__((ext_vector_type(4)));

constexpr int WIN_MAX_RUNS = 16;      // window length up to 2048 steps held in registers

// one workgroup per (new entry, head); threads stride over the medoids
__global__ __launch_bounds__(256) void window_count_kernel(const v4u* __restrict__ bits, int nruns, int Npad, int N, int W,
                                                           const int32_t* __restrict__ new_ids, int n_new,
                                                           const int32_t* __restrict__ medoids, int Nc, double tau,
                                                           int32_t* __restrict__ f_out, uint8_t* __restrict__ member,
                                                           uint32_t* __restrict__ dev_flags) {
    const int a = blockIdx.x, h = blockIdx.y;
    const int32_t e = new_ids[(size_t)h * n_new + a];
    const bool e_ok = e >= 0 && e < N;
    const v4u* hb = bits + (size_t)h * nruns * Npad;
    v4u mine[WIN_MAX_RUNS];
#pragma unroll
    for (int r = 0; r < WIN_MAX_RUNS; ++r) {
        mine[r] = v4u{0u, 0u, 0u, 0u};
        if (r < nruns && e_ok) mine[r] = hb[(size_t)r * Npad + e];
    }
    bool bad = !e_ok;
    for (int c = threadIdx.x; c < Nc; c += 256) {
        const int32_t m = medoids[(size_t)h * Nc + c];
        int32_t f = 0;
        if (m >= 0 && m < N) {
#pragma unroll
            for (int r = 0; r < WIN_MAX_RUNS; ++r)
                if (r < nruns) {
                    const v4u o = hb[(size_t)r * Npad + m];
                    f += __popc(mine[r].x & o.x) + __popc(mine[r].y & o.y) + __popc(mine[r].z & o.z) + __popc(mine[r].w & o.w);
                }
        } else {
            bad = true;
        }
        const double d = 1.0 - (double)f / (double)W;
        const size_t o = ((size_t)h * n_new + a) * Nc + c;
        if (f_out) f_out[o] = f;
        member[o] = d < tau ? 1 : 0;
    }
    if (bad) atomicOr(dev_flags, SWARM_DEV_BAD_ENTRY);
}

// one thread per (cluster, head): walks the new entries in order, the cluster grows as they join
__global__ void window_place_kernel(const uint8_t* __restrict__ member, int n_new, int Nc, const int32_t* __restrict__ primary,
                                    const int32_t* __restrict__ size, int D, int32_t* __restrict__ disk) {
    const int c = blockIdx.x * blockDim.x + threadIdx.x, h = blockIdx.y;
    if (c >= Nc) return;
    const int64_t base = (int64_t)primary[(size_t)h * Nc + c] + size[(size_t)h * Nc + c] + 1;
    int64_t grown = 0;
    for (int a = 0; a < n_new; ++a) {
        const size_t o = ((size_t)h * n_new + a) * Nc + c;
        int32_t v = -1;
        if (member[o]) { v = (int32_t)((base + grown) % D); ++grown; }
        disk[o] = v;
    }
}

}  // namespace

swarm_status launch_window(swarm_ctx* ctx, int nruns, int Npad, int N, int W, int H, const int32_t* new_ids, int n_new,
                           const int32_t* medoids, int Nc, double tau, const int32_t* primary, const int32_t* size, int D,
                           int32_t* f_out, uint8_t* member, int32_t* disk) {
    hipLaunchKernelGGL(window_count_kernel, dim3((unsigned)n_new, (unsigned)H), dim3(256), 0, ctx->stream,
                       reinterpret_cast<const v4u*>(ctx->trace), nruns, Npad, N, W, new_ids, n_new, medoids, Nc, tau, f_out,
                       member, ctx->dev_flags);
    swarm_status st = swarm_check_launch(ctx, "window_count_kernel");
    if (st != SWARM_OK || !disk) return st;
    hipLaunchKernelGGL(window_place_kernel, dim3((unsigned)((Nc + 127) / 128), (unsigned)H), dim3(128), 0, ctx->stream, member,
                       n_new, Nc, primary, size, D, disk);
    return swarm_check_launch(ctx, "window_place_kernel");
}
