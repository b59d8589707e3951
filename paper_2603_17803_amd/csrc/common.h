// Internal declarations shared by the translation units of libswarm (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include <utility>
#include <vector>

#include "swarm.h"

struct swarm_graph {
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
};

struct swarm_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    char err[512] = {0};

    // scratch, grown on demand
    float* scores = nullptr;       // [B][H][N] when the caller passes no score buffer
    int32_t* cand = nullptr;       // winners of the slices of long rows (two-stage selection)
    size_t cand_bytes = 0;
    size_t scores_bytes = 0;
    void* trace = nullptr;         // binary trace as bits: uint4 [H][runs of 128 rows][Npad]
    size_t trace_bytes = 0;
    int64_t* totals = nullptr;     // per-head grand totals of C when the caller keeps none
    size_t totals_bytes = 0;
    bool trace_lds_opt_in = false, syrk_lds_opt_in = false, batched_lds_opt_in = false;   // large dynamic LDS enabled for this context's device
    uint32_t* dev_flags = nullptr; // sticky SWARM_DEV_* bits (one word)
    void* static_scratch = nullptr; // this device's copy of the library's static scratch array (address resolved at create)
    std::vector<std::pair<int, int32_t*>> tile_orders;   // co-activation tile schedules, one per tile count, never rewritten
    bool capturing = false;
    bool recorded = false;         // a graph has been recorded on this context: it may refer to any scratch address
    std::vector<void*> retired;    // outgrown scratch that recorded graphs may still use; freed with the context
};

#define SWARM_HIP(ctx, call)                                                                      \
    do {                                                                                          \
        hipError_t e_ = (call);                                                                   \
        if (e_ != hipSuccess) {                                                                   \
            snprintf((ctx)->err, sizeof((ctx)->err), "%s failed: %s (%s:%d)", #call,              \
                     hipGetErrorString(e_), __FILE__, __LINE__);                                  \
            return SWARM_EHIP;                                                                    \
        }                                                                                         \
    } while (0)

#define SWARM_REJECT(ctx, ...)                                                                    \
    do {                                                                                          \
        snprintf((ctx)->err, sizeof((ctx)->err), __VA_ARGS__);                                    \
        return SWARM_EINVAL;                                                                      \
    } while (0)

// First statement of every entry point: a context is required, and its device must be the calling
// thread's current device (kernels and allocations go to the current device).
#define SWARM_ENTER(ctx)                                                                          \
    do {                                                                                          \
        if (!(ctx)) return SWARM_EINVAL;                                                          \
        int cur_ = -1;                                                                            \
        if (hipGetDevice(&cur_) != hipSuccess || cur_ != (ctx)->device)                           \
            SWARM_REJECT(ctx, "the context belongs to device %d but device %d is current", (ctx)->device, cur_); \
    } while (0)

// Argument checks shared by the scoring entry points.
swarm_status swarm_check_score_args(swarm_ctx* ctx, const char* fn, const swarm_keys* keys, const void* q, int32_t B);
// Resolves this device's copy of the library's static scratch (called by swarm_create with the device current).
swarm_status swarm_static_scratch_init(swarm_ctx* ctx);
size_t select_cand_bytes(int64_t rows, int N, int k);           // scratch the sliced selection needs for its winners (0: not sliced)

// Grows a scratch buffer to at least `bytes` (never shrinks).  Allocation synchronises the stream.
swarm_status swarm_grow(swarm_ctx* ctx, void** buf, size_t* have, size_t bytes);

// Fixed scratch handed to the launchers in place of the context's growing buffers (for the entry point that
// may not allocate): the winners of the sliced selection.
struct swarm_fixed_scratch {
    int32_t* cand;
    size_t cand_bytes;
};

// --- kernel launchers (each enqueues on ctx->stream and reports launch errors) ---------------
constexpr int SWARM_BATCHED_MIN_STREAMS = 8;   // from this many streams on, scoring runs as a GEMM on the matrix cores
swarm_status launch_score(swarm_ctx* ctx, const swarm_keys* keys, const void* q, int B, float* scores,
                          const int32_t* row_ids = nullptr, int M = 0);
swarm_status launch_select(swarm_ctx* ctx, const float* scores, int64_t rows, int N, int k, int32_t* out_idx,
                           const swarm_fixed_scratch* fixed = nullptr);
bool select_uses_slices(int64_t rows, int N, int k);   // long rows, few of them: sliced two-stage selection
swarm_status launch_select_slices(swarm_ctx* ctx, const float* scores, int64_t rows, int N, int k, int* M_out, int* stride_out,
                                  int32_t** cand_out, const swarm_fixed_scratch* fixed = nullptr);
swarm_status launch_trace_build(swarm_ctx* ctx, const int32_t* idx, int64_t rows, int H, int k, int N, int Npad,
                                int nruns, uint32_t flags, int32_t* row_count = nullptr);   // row_count: int32 [H][nruns*128] out, optional
swarm_status launch_trace_totals_thresholds(swarm_ctx* ctx, const int32_t* row_count, int H, int nrows, double tau, uint32_t flags,
                                            int64_t* totals, int64_t* cstar);
swarm_status launch_fill_i32(swarm_ctx* ctx, int32_t* p, size_t n, int32_t v);
swarm_status launch_coact_syrk(swarm_ctx* ctx, int H, int N, int Npad, int nruns, int32_t* C, uint32_t decay_q16,
                               const int64_t* cstar = nullptr, int32_t* rho = nullptr);
swarm_status launch_rho_exclude_self(swarm_ctx* ctx, const int32_t* C, int H, int N, const int64_t* cstar, int32_t* rho);
swarm_status launch_medoid_rank(swarm_ctx* ctx, const int32_t* rho, int H, int N, int32_t* queue);
swarm_status launch_coact_popcount(swarm_ctx* ctx, int H, int N, int Npad, int nruns, int32_t* C, uint32_t decay_q16);
size_t map_lds_base_bytes(int Nc, int cap);   // on-chip staging of the mapping step before any table is staged
swarm_status launch_map(swarm_ctx* ctx, const int32_t* sel, int64_t groups, int S, int H, int N, const int32_t* e2c,
                        int Nc, const int32_t* replicas, int R, int D, const int32_t* weight,
                        const uint32_t* resident, int32_t* q_off, int32_t* q_cluster, int32_t* q_load, int cap, int piece = 0);
swarm_status launch_density(swarm_ctx* ctx, const int32_t* C, int H, int N, const int64_t* totals_in, double tau,
                            uint32_t flags, int32_t* rho, int32_t* queue, int64_t* totals);
swarm_status launch_window(swarm_ctx* ctx, int nruns, int Npad, int N, int W, int H, const int32_t* new_ids, int n_new,
                           const int32_t* medoids, int Nc, double tau, const int32_t* primary, const int32_t* size, int D,
                           int32_t* f_out, uint8_t* member, int32_t* disk);
swarm_status launch_expand_clusters(swarm_ctx* ctx, const int32_t* clusters, int64_t groups, int Sc, int H, int Nc,
                                    const int32_t* cl_off, const int32_t* cl_entries, int E, int32_t* entries, int32_t* count,
                                    int cap_e);
swarm_status launch_submission_order(swarm_ctx* ctx, const int32_t* q_off, const int32_t* q_cluster, int64_t groups, int D, int cap,
                                     int32_t* order, int32_t* batch_off, int32_t* nb);
swarm_status launch_select_map(swarm_ctx* ctx, const float* scores, int H, int N, int k, int32_t* out_idx,
                               const int32_t* e2c, int Nc, const int32_t* replicas, int R, int D, const int32_t* weight,
                               const uint32_t* resident, int32_t* q_off, int32_t* q_cluster, int32_t* q_load, int cap,
                               bool* launched);

static inline swarm_status swarm_check_launch(swarm_ctx* ctx, const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        snprintf(ctx->err, sizeof(ctx->err), "launch of %s failed: %s", what, hipGetErrorString(e));
        return SWARM_EHIP;
    }
    return SWARM_OK;
}
