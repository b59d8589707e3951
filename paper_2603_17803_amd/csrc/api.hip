// C-ABI entry points of libswarm: argument validation, scratch management, kernel sequencing.
// Every step of the path runs in the HIP kernels of the sibling files; nothing here computes.
#include <new>
#include <string.h>

#include "common.h"

static char g_create_err[512] = "";

swarm_status swarm_grow(swarm_ctx* ctx, void** buf, size_t* have, size_t bytes) {
    if (*have >= bytes) return SWARM_OK;
    if (ctx->capturing) {
        snprintf(ctx->err, sizeof(ctx->err), "scratch must grow to %zu bytes while recording; run the sequence once first", bytes);
        return SWARM_EINVAL;
    }
    SWARM_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (*buf) {
        if (ctx->recorded) {
            // a recorded graph may replay kernels that use the old buffer: keep it until the context goes
            try {
                ctx->retired.push_back(*buf);
            } catch (...) {
                snprintf(ctx->err, sizeof(ctx->err), "out of host memory");
                return SWARM_ENOMEM;
            }
        } else {
            SWARM_HIP(ctx, hipFree(*buf));
        }
    }
    *buf = nullptr;
    *have = 0;
    hipError_t e = hipMalloc(buf, bytes);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        snprintf(ctx->err, sizeof(ctx->err), "scratch allocation of %zu bytes failed: %s", bytes, hipGetErrorString(e));
        *buf = nullptr;
        return SWARM_ENOMEM;
    }
    *have = bytes;
    return SWARM_OK;
}

extern "C" {

swarm_status swarm_create(swarm_ctx** out, int device, void* hip_stream) {
    if (!out) return SWARM_EINVAL;
    *out = nullptr;
    int ndev = 0;
    hipError_t e = hipGetDeviceCount(&ndev);
    if (e != hipSuccess || device < 0 || device >= ndev) {
        snprintf(g_create_err, sizeof g_create_err, "no HIP device %d (count %d, %s)", device, ndev,
                 hipGetErrorString(e));
        (void)hipGetLastError();
        return e != hipSuccess ? SWARM_EHIP : SWARM_EINVAL;
    }
    hipDeviceProp_t prop;
    e = hipSetDevice(device);
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, device);
    if (e != hipSuccess) {
        snprintf(g_create_err, sizeof g_create_err, "cannot query device %d: %s", device, hipGetErrorString(e));
        return SWARM_EHIP;
    }
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0) {
        snprintf(g_create_err, sizeof g_create_err, "device %d is %s; this library is built for gfx950 only", device,
                 prop.gcnArchName);
        return SWARM_EINVAL;
    }
    swarm_ctx* ctx = new (std::nothrow) swarm_ctx();
    if (!ctx) {
        snprintf(g_create_err, sizeof g_create_err, "out of host memory");
        return SWARM_ENOMEM;
    }
    ctx->device = device;
    ctx->stream = static_cast<hipStream_t>(hip_stream);
    if (swarm_static_scratch_init(ctx) != SWARM_OK) {
        snprintf(g_create_err, sizeof g_create_err, "%s", ctx->err);
        delete ctx;
        return SWARM_EHIP;
    }
    e = hipMalloc(reinterpret_cast<void**>(&ctx->dev_flags), 256);
    if (e == hipSuccess) e = hipMemsetAsync(ctx->dev_flags, 0, 256, ctx->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
    if (e != hipSuccess) {
        snprintf(g_create_err, sizeof g_create_err, "context set-up failed: %s", hipGetErrorString(e));
        delete ctx;
        return SWARM_EHIP;
    }
    *out = ctx;
    return SWARM_OK;
}

swarm_status swarm_destroy(swarm_ctx* ctx) {
    if (!ctx) return SWARM_EINVAL;
    (void)hipStreamSynchronize(ctx->stream);
    if (ctx->scores) (void)hipFree(ctx->scores);
    if (ctx->trace) (void)hipFree(ctx->trace);
    if (ctx->cand) (void)hipFree(ctx->cand);
    if (ctx->totals) (void)hipFree(ctx->totals);
    for (auto& t : ctx->tile_orders) (void)hipFree(t.second);
    for (void* p : ctx->retired) (void)hipFree(p);
    if (ctx->dev_flags) (void)hipFree(ctx->dev_flags);
    delete ctx;
    return SWARM_OK;
}

const char* swarm_last_error(const swarm_ctx* ctx) { return ctx ? ctx->err : g_create_err; }

#ifndef SWARM_SOURCE_HASH
#define SWARM_SOURCE_HASH "unknown"
#endif
const char* swarm_source_hash(void) { return SWARM_SOURCE_HASH; }

swarm_status swarm_device_status(swarm_ctx* ctx, uint32_t* flags) {
    SWARM_ENTER(ctx);
    if (ctx->capturing) SWARM_REJECT(ctx, "device_status: not while recording");
    uint32_t host = 0;
    SWARM_HIP(ctx, hipMemcpyAsync(&host, ctx->dev_flags, sizeof host, hipMemcpyDeviceToHost, ctx->stream));
    SWARM_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (host) {
        SWARM_HIP(ctx, hipMemsetAsync(ctx->dev_flags, 0, sizeof host, ctx->stream));
        SWARM_HIP(ctx, hipStreamSynchronize(ctx->stream));
    }
    if (flags) *flags = host;
    if (host) {
        snprintf(ctx->err, sizeof(ctx->err), "device data flags 0x%x", host);
        return SWARM_EDATA;
    }
    return SWARM_OK;
}

}  // extern "C"

swarm_status swarm_check_score_args(swarm_ctx* ctx, const char* fn, const swarm_keys* keys, const void* q, int32_t B) {
    if (!keys || !keys->data || !q) SWARM_REJECT(ctx, "%s: NULL keys, data or q", fn);
    if (keys->kind != SWARM_KEYS_TOKEN && keys->kind != SWARM_KEYS_PAGE_MINMAX)
        SWARM_REJECT(ctx, "%s: unknown key kind %d", fn, keys->kind);
    if (keys->H < 1 || keys->N < 1 || keys->G < 1 || B < 1)
        SWARM_REJECT(ctx, "%s: H=%d N=%d G=%d B=%d must all be >= 1", fn, keys->H, keys->N, keys->G, B);
    if (keys->d < 8 || keys->d % 8 != 0 || keys->d > 512)
        SWARM_REJECT(ctx, "%s: d=%d must be a multiple of 8 in [8,512]", fn, keys->d);
    if ((reinterpret_cast<uintptr_t>(keys->data) & 15) || (reinterpret_cast<uintptr_t>(q) & 15))
        SWARM_REJECT(ctx, "%s: keys.data and q must be 16-byte aligned", fn);
    if ((int64_t)B * keys->H > (int64_t)1 << 24) SWARM_REJECT(ctx, "%s: B*H too large", fn);
    if (keys->N > (1 << 30) || keys->H > 65535) SWARM_REJECT(ctx, "%s: N=%d above 2^30 or H=%d above 65535", fn, keys->N, keys->H);
    return SWARM_OK;
}

extern "C" {

swarm_status swarm_score(swarm_ctx* ctx, const swarm_keys* keys, const void* q, int32_t B, float* out_scores) {
    SWARM_ENTER(ctx);
    swarm_status st = swarm_check_score_args(ctx, "score", keys, q, B);
    if (st != SWARM_OK) return st;
    if (!out_scores || (reinterpret_cast<uintptr_t>(out_scores) & 3)) SWARM_REJECT(ctx, "score: NULL or misaligned out_scores");
    return launch_score(ctx, keys, q, B, out_scores);
}

swarm_status swarm_score_select(swarm_ctx* ctx, const swarm_keys* keys, const void* q, int32_t B, int32_t k,
                                int32_t* out_idx, float* out_scores) {
    SWARM_ENTER(ctx);
    swarm_status st = swarm_check_score_args(ctx, "score_select", keys, q, B);
    if (st != SWARM_OK) return st;
    if (!out_idx) SWARM_REJECT(ctx, "score_select: NULL out_idx");
    if (k < 1 || k > keys->N) SWARM_REJECT(ctx, "score_select: k=%d outside [1,N=%d]", k, keys->N);
    if (out_scores && (reinterpret_cast<uintptr_t>(out_scores) & 3)) SWARM_REJECT(ctx, "score_select: out_scores misaligned");

    float* scores = out_scores;
    if (!scores) {
        st = swarm_grow(ctx, reinterpret_cast<void**>(&ctx->scores), &ctx->scores_bytes,
                        sizeof(float) * (size_t)B * keys->H * keys->N);
        if (st != SWARM_OK) return st;
        scores = ctx->scores;
    }
    st = launch_score(ctx, keys, q, B, scores);
    if (st != SWARM_OK) return st;
    return launch_select(ctx, scores, (int64_t)B * keys->H, keys->N, k, out_idx);
}

swarm_status swarm_score_select_indexed(swarm_ctx* ctx, const swarm_keys* keys, const int32_t* row_ids, int32_t M, const void* q,
                                        int32_t B, int32_t k, int32_t* out_idx, float* out_scores) {
    SWARM_ENTER(ctx);
    swarm_status st = swarm_check_score_args(ctx, "score_select_indexed", keys, q, B);
    if (st != SWARM_OK) return st;
    if (!row_ids || !out_idx) SWARM_REJECT(ctx, "score_select_indexed: NULL row_ids or out_idx");
    if (M < 1) SWARM_REJECT(ctx, "score_select_indexed: M=%d must be >= 1", M);
    if (k < 1 || k > M) SWARM_REJECT(ctx, "score_select_indexed: k=%d outside [1,M=%d]", k, M);
    if (out_scores && (reinterpret_cast<uintptr_t>(out_scores) & 3)) SWARM_REJECT(ctx, "score_select_indexed: out_scores misaligned");
    float* scores = out_scores;
    if (!scores) {
        st = swarm_grow(ctx, reinterpret_cast<void**>(&ctx->scores), &ctx->scores_bytes, sizeof(float) * (size_t)B * keys->H * M);
        if (st != SWARM_OK) return st;
        scores = ctx->scores;
    }
    st = launch_score(ctx, keys, q, B, scores, row_ids, M);
    if (st != SWARM_OK) return st;
    return launch_select(ctx, scores, (int64_t)B * keys->H, M, k, out_idx);
}

swarm_status swarm_expand_clusters(swarm_ctx* ctx, const int32_t* clusters, int64_t groups, int32_t Sc, int32_t H, int32_t Nc,
                                   const int32_t* cl_off, const int32_t* cl_entries, int32_t E, int32_t* entries, int32_t* count,
                                   int32_t cap_e) {
    SWARM_ENTER(ctx);
    if (!clusters || !cl_off || !cl_entries || !entries || !count) SWARM_REJECT(ctx, "expand_clusters: NULL required pointer");
    if (groups < 1 || groups > ((int64_t)1 << 30) || Sc < 1 || H < 1 || Nc < 1 || E < 1 || cap_e < 1)
        SWARM_REJECT(ctx, "expand_clusters: groups=%lld Sc=%d H=%d Nc=%d E=%d cap_e=%d must all be >= 1", (long long)groups, Sc,
                     H, Nc, E, cap_e);
    if (Nc > (1 << 18)) SWARM_REJECT(ctx, "expand_clusters: Nc=%d above 2^18", Nc);
    return launch_expand_clusters(ctx, clusters, groups, Sc, H, Nc, cl_off, cl_entries, E, entries, count, cap_e);
}

swarm_status swarm_submission_order(swarm_ctx* ctx, const int32_t* q_off, const int32_t* q_cluster, int64_t groups, int32_t D,
                                    int32_t cap, int32_t* order, int32_t* batch_off, int32_t* nb) {
    SWARM_ENTER(ctx);
    if (!q_off || !q_cluster || !order || !batch_off || !nb) SWARM_REJECT(ctx, "submission_order: NULL required pointer");
    if (groups < 1 || groups > ((int64_t)1 << 30) || D < 1 || D > 64 || cap < 1)
        SWARM_REJECT(ctx, "submission_order: groups=%lld D=%d cap=%d out of range", (long long)groups, D, cap);
    return launch_submission_order(ctx, q_off, q_cluster, groups, D, cap, order, batch_off, nb);
}

static swarm_status check_coact_args(swarm_ctx* ctx, const char* fn, const int32_t* idx, int64_t rows, int32_t H, int32_t k,
                                     int32_t N, const int32_t* C, uint32_t flags, uint32_t allowed_flags) {
    if (!idx || !C) SWARM_REJECT(ctx, "%s: NULL idx or C", fn);
    if (H < 1 || N < 1 || k < 1 || k > N) SWARM_REJECT(ctx, "%s: H=%d N=%d k=%d invalid", fn, H, N, k);
    if (N > (1 << 20) || H > 65535) SWARM_REJECT(ctx, "%s: N=%d above 2^20 or H=%d above 65535", fn, N, H);
    if (rows < 1 || rows > ((int64_t)1 << 24)) SWARM_REJECT(ctx, "%s: rows=%lld outside [1,2^24]", fn, (long long)rows);
    if (flags & ~allowed_flags) SWARM_REJECT(ctx, "%s: unknown flags 0x%x", fn, flags);
    if ((flags & SWARM_CHECK_IDX) && rows * H > ((int64_t)1 << 30))
        SWARM_REJECT(ctx, "%s: SWARM_CHECK_IDX handles at most 2^30 (row, head) selections per call", fn);
    if (reinterpret_cast<uintptr_t>(C) & 15) SWARM_REJECT(ctx, "%s: C must be 16-byte aligned", fn);
    return SWARM_OK;
}

swarm_status swarm_coact_accumulate(swarm_ctx* ctx, const int32_t* idx, int64_t rows, int32_t H, int32_t k,
                                    int32_t N, int32_t* C, uint32_t decay_q16, uint32_t flags) {
    SWARM_ENTER(ctx);
    swarm_status st = check_coact_args(ctx, "coact_accumulate", idx, rows, H, k, N, C, flags, SWARM_CHECK_IDX | SWARM_COACT_POPCOUNT);
    if (st != SWARM_OK) return st;
    if (decay_q16 > 65536u) SWARM_REJECT(ctx, "coact_accumulate: decay_q16=%u above 65536", decay_q16);

    const int nruns = (int)((rows + 511) / 512 * 4);      // contraction in runs of 128 trace rows, zero-padded to a multiple of 4 runs
    const int Npad = (N + 255) / 256 * 256;               // entries, zero-padded to the C tile
    st = swarm_grow(ctx, &ctx->trace, &ctx->trace_bytes, (size_t)H * nruns * Npad * 16);
    if (st != SWARM_OK) return st;
    st = launch_trace_build(ctx, idx, rows, H, k, N, Npad, nruns, flags);
    if (st != SWARM_OK) return st;
    if (flags & SWARM_COACT_POPCOUNT) return launch_coact_popcount(ctx, H, N, Npad, nruns, C, decay_q16);
    return launch_coact_syrk(ctx, H, N, Npad, nruns, C, decay_q16);
}

swarm_status swarm_coact_build_density(swarm_ctx* ctx, const int32_t* idx, int64_t rows, int32_t H, int32_t k, int32_t N,
                                       int32_t* C, uint32_t flags, double tau, uint32_t rho_flags, int32_t* rho, int32_t* queue,
                                       int64_t* totals_out) {
    SWARM_ENTER(ctx);
    swarm_status st = check_coact_args(ctx, "coact_build_density", idx, rows, H, k, N, C, flags, SWARM_CHECK_IDX);
    if (st != SWARM_OK) return st;
    if (!rho) SWARM_REJECT(ctx, "coact_build_density: NULL rho");
    if (rho_flags & ~(SWARM_RHO_EXCLUDE_SELF | SWARM_RHO_STRICT)) SWARM_REJECT(ctx, "coact_build_density: unknown rho_flags 0x%x", rho_flags);
    if (totals_out && (reinterpret_cast<uintptr_t>(totals_out) & 7)) SWARM_REJECT(ctx, "coact_build_density: totals_out must be 8-byte aligned");

    const int nruns = (int)((rows + 511) / 512 * 4);
    const int Npad = (N + 255) / 256 * 256;
    st = swarm_grow(ctx, &ctx->trace, &ctx->trace_bytes, (size_t)H * nruns * Npad * 16);
    if (st != SWARM_OK) return st;
    // auxiliary scratch: totals [H] and thresholds [H] (int64), then the trace rows' entry counts [H][nruns * 128] (int32)
    st = swarm_grow(ctx, reinterpret_cast<void**>(&ctx->totals), &ctx->totals_bytes,
                    sizeof(int64_t) * 2 * (size_t)H + sizeof(int32_t) * (size_t)H * nruns * 128);
    if (st != SWARM_OK) return st;
    int64_t* totals = totals_out ? totals_out : ctx->totals;
    int64_t* cstar = ctx->totals + H;
    int32_t* row_count = reinterpret_cast<int32_t*>(ctx->totals + 2 * (size_t)H);

    if (N & 3) {
        // rows of C are not 16-byte aligned: the epilogue has no vector pass to count in; build, then sweep
        st = launch_trace_build(ctx, idx, rows, H, k, N, Npad, nruns, flags);
        if (st == SWARM_OK) st = launch_coact_syrk(ctx, H, N, Npad, nruns, C, 0u);
        if (st != SWARM_OK) return st;
        return launch_density(ctx, C, H, N, nullptr, tau, rho_flags, rho, queue, totals);
    }
    st = launch_trace_build(ctx, idx, rows, H, k, N, Npad, nruns, flags, row_count);
    if (st == SWARM_OK) st = launch_trace_totals_thresholds(ctx, row_count, H, nruns * 128, tau, rho_flags, totals, cstar);
    if (st == SWARM_OK) st = launch_fill_i32(ctx, rho, (size_t)H * N, 0);
    if (st == SWARM_OK) st = launch_coact_syrk(ctx, H, N, Npad, nruns, C, 0u, cstar, rho);
    if (st == SWARM_OK && (rho_flags & SWARM_RHO_EXCLUDE_SELF)) st = launch_rho_exclude_self(ctx, C, H, N, cstar, rho);
    if (st == SWARM_OK && queue) st = launch_medoid_rank(ctx, rho, H, N, queue);
    return st;
}

swarm_status swarm_coact_density(swarm_ctx* ctx, const int32_t* C, int32_t H, int32_t N, const int64_t* totals_in,
                                 double tau, uint32_t flags, int32_t* rho, int32_t* queue, int64_t* totals_out) {
    SWARM_ENTER(ctx);
    if (!C || !rho) SWARM_REJECT(ctx, "coact_density: NULL C or rho");
    if (H < 1 || N < 1) SWARM_REJECT(ctx, "coact_density: H=%d N=%d must be >= 1", H, N);
    if (N > (1 << 20) || H > 65535) SWARM_REJECT(ctx, "coact_density: N=%d above 2^20 or H=%d above 65535", N, H);
    if (reinterpret_cast<uintptr_t>(C) & 15) SWARM_REJECT(ctx, "coact_density: C must be 16-byte aligned");
    if (flags & ~(SWARM_RHO_EXCLUDE_SELF | SWARM_RHO_STRICT)) SWARM_REJECT(ctx, "coact_density: unknown flags 0x%x", flags);
    if ((totals_in && (reinterpret_cast<uintptr_t>(totals_in) & 7)) || (totals_out && (reinterpret_cast<uintptr_t>(totals_out) & 7)))
        SWARM_REJECT(ctx, "coact_density: totals must be 8-byte aligned");
    int64_t* totals = totals_out;
    if (!totals) {
        const swarm_status st = swarm_grow(ctx, reinterpret_cast<void**>(&ctx->totals), &ctx->totals_bytes, sizeof(int64_t) * (size_t)H);
        if (st != SWARM_OK) return st;
        totals = ctx->totals;
    }
    return launch_density(ctx, C, H, N, totals_in, tau, flags, rho, queue, totals);
}

swarm_status swarm_window_assign(swarm_ctx* ctx, const int32_t* sel, int32_t W, int32_t H, int32_t k, int32_t N,
                                 const int32_t* new_ids, int32_t n_new, const int32_t* medoids, int32_t Nc, double tau,
                                 const int32_t* primary, const int32_t* size, int32_t D, int32_t* f_out, uint8_t* member,
                                 int32_t* disk) {
    SWARM_ENTER(ctx);
    if (!sel || !new_ids || !medoids || !member) SWARM_REJECT(ctx, "window_assign: NULL required pointer");
    if (W < 1 || W > 2048) SWARM_REJECT(ctx, "window_assign: W=%d outside [1,2048]", W);
    if (H < 1 || N < 1 || k < 1 || k > N || n_new < 1 || Nc < 1)
        SWARM_REJECT(ctx, "window_assign: H=%d N=%d k=%d n_new=%d Nc=%d invalid", H, N, k, n_new, Nc);
    if (N > (1 << 24) || H > 65535) SWARM_REJECT(ctx, "window_assign: N=%d above 2^24 or H=%d above 65535", N, H);
    if ((primary == nullptr) != (size == nullptr)) SWARM_REJECT(ctx, "window_assign: primary and size go together");
    if (disk && (!primary || D < 1)) SWARM_REJECT(ctx, "window_assign: disk needs primary, size and D >= 1");
    const int nruns = (W + 127) / 128;
    const int Npad = (N + 255) / 256 * 256;
    swarm_status st = swarm_grow(ctx, &ctx->trace, &ctx->trace_bytes, (size_t)H * nruns * Npad * 16);
    if (st != SWARM_OK) return st;
    st = launch_trace_build(ctx, sel, W, H, k, N, Npad, nruns, 0u);
    if (st != SWARM_OK) return st;
    return launch_window(ctx, nruns, Npad, N, W, H, new_ids, n_new, medoids, Nc, tau, primary, size, D, f_out, member, disk);
}

static swarm_status check_map_args(swarm_ctx* ctx, const char* fn, int64_t groups, int32_t S, int32_t H, int32_t N,
                                   const int32_t* e2c, int32_t Nc, const int32_t* replicas, int32_t R, int32_t D,
                                   const int32_t* q_off, const int32_t* q_cluster, const int32_t* q_load, int32_t cap) {
    if (!e2c || !replicas || !q_off || !q_cluster || !q_load) SWARM_REJECT(ctx, "%s: NULL required pointer", fn);
    if (groups < 1 || groups > ((int64_t)1 << 30) || S < 1 || H < 1 || N < 1 || Nc < 1 || cap < 1)
        SWARM_REJECT(ctx, "%s: groups=%lld S=%d H=%d N=%d Nc=%d cap=%d must all be >= 1", fn, (long long)groups, S, H, N,
                     Nc, cap);
    if (R < 1 || R > D || D > 64) SWARM_REJECT(ctx, "%s: need 1 <= R=%d <= D=%d <= 64", fn, R, D);
    if (Nc > (1 << 20)) SWARM_REJECT(ctx, "%s: Nc=%d above 2^20", fn, Nc);
    const size_t lds = map_lds_base_bytes(Nc, cap);
    if (lds > 64u * 1024u)
        SWARM_REJECT(ctx, "%s: cap=%d and Nc=%d need %zu bytes of on-chip staging (limit 64 KiB)", fn, cap, Nc, lds);
    return SWARM_OK;
}

swarm_status swarm_map_requests(swarm_ctx* ctx, const int32_t* sel, int64_t groups, int32_t S, int32_t H, int32_t N,
                                const int32_t* e2c, int32_t Nc, const int32_t* replicas, int32_t R, int32_t D,
                                const int32_t* weight, const uint32_t* resident,
                                int32_t* q_off, int32_t* q_cluster, int32_t* q_load, int32_t cap) {
    SWARM_ENTER(ctx);
    if (!sel) SWARM_REJECT(ctx, "map_requests: NULL sel");
    const swarm_status st = check_map_args(ctx, "map_requests", groups, S, H, N, e2c, Nc, replicas, R, D, q_off, q_cluster,
                                           q_load, cap);
    if (st != SWARM_OK) return st;
    return launch_map(ctx, sel, groups, S, H, N, e2c, Nc, replicas, R, D, weight, resident, q_off, q_cluster, q_load,
                      cap);
}

swarm_status swarm_map_requests_streams(swarm_ctx* ctx, const int32_t* idx, int64_t steps, int32_t B, int32_t H, int32_t k, int32_t N,
                                        const int32_t* e2c, int32_t Nc, const int32_t* replicas, int32_t R, int32_t D,
                                        const int32_t* weight, const uint32_t* resident,
                                        int32_t* q_off, int32_t* q_cluster, int32_t* q_load, int32_t cap) {
    SWARM_ENTER(ctx);
    if (!idx) SWARM_REJECT(ctx, "map_requests_streams: NULL idx");
    if (steps < 1 || B < 1 || k < 1 || H < 1) SWARM_REJECT(ctx, "map_requests_streams: steps=%lld B=%d H=%d k=%d must all be >= 1", (long long)steps, B, H, k);
    if ((int64_t)B * k > ((int64_t)1 << 24) || (int64_t)H * k > ((int64_t)1 << 30) || steps * H > ((int64_t)1 << 30))
        SWARM_REJECT(ctx, "map_requests_streams: B*k above 2^24, H*k above 2^30 or steps*H above 2^30");
    const swarm_status st = check_map_args(ctx, "map_requests_streams", steps * H, B * k, H, N, e2c, Nc, replicas, R, D, q_off, q_cluster,
                                           q_load, cap);
    if (st != SWARM_OK) return st;
    return launch_map(ctx, idx, steps * H, B * k, H, N, e2c, Nc, replicas, R, D, weight, resident, q_off, q_cluster, q_load, cap, k);
}

swarm_status swarm_step(swarm_ctx* ctx, const swarm_keys* keys, const void* q, int32_t k, int32_t* out_idx,
                        float* out_scores, const int32_t* e2c, int32_t Nc, const int32_t* replicas, int32_t R, int32_t D,
                        const int32_t* weight, const uint32_t* resident, int32_t* q_off, int32_t* q_cluster,
                        int32_t* q_load, int32_t cap) {
    SWARM_ENTER(ctx);
    swarm_status st = swarm_check_score_args(ctx, "step", keys, q, 1);
    if (st != SWARM_OK) return st;
    if (!out_idx) SWARM_REJECT(ctx, "step: NULL out_idx");
    if (k < 1 || k > keys->N) SWARM_REJECT(ctx, "step: k=%d outside [1,N=%d]", k, keys->N);
    if (out_scores && (reinterpret_cast<uintptr_t>(out_scores) & 3)) SWARM_REJECT(ctx, "step: out_scores misaligned");
    st = check_map_args(ctx, "step", keys->H, k, keys->H, keys->N, e2c, Nc, replicas, R, D, q_off, q_cluster, q_load, cap);
    if (st != SWARM_OK) return st;

    float* scores = out_scores;
    if (!scores) {
        st = swarm_grow(ctx, reinterpret_cast<void**>(&ctx->scores), &ctx->scores_bytes,
                        sizeof(float) * (size_t)keys->H * keys->N);
        if (st != SWARM_OK) return st;
        scores = ctx->scores;
    }
    st = launch_score(ctx, keys, q, 1, scores);
    if (st != SWARM_OK) return st;
    bool fused = false;
    st = launch_select_map(ctx, scores, keys->H, keys->N, k, out_idx, e2c, Nc, replicas, R, D, weight, resident, q_off,
                           q_cluster, q_load, cap, &fused);
    if (st != SWARM_OK || fused) return st;
    st = launch_select(ctx, scores, keys->H, keys->N, k, out_idx);
    if (st != SWARM_OK) return st;
    return launch_map(ctx, out_idx, keys->H, k, keys->H, keys->N, e2c, Nc, replicas, R, D, weight, resident, q_off,
                      q_cluster, q_load, cap);
}

swarm_status swarm_capture_begin(swarm_ctx* ctx) {
    SWARM_ENTER(ctx);
    if (ctx->capturing) SWARM_REJECT(ctx, "capture_begin: already recording");
    if (!ctx->stream) SWARM_REJECT(ctx, "capture_begin: the NULL stream cannot be recorded");
    SWARM_HIP(ctx, hipStreamBeginCapture(ctx->stream, hipStreamCaptureModeThreadLocal));
    ctx->capturing = true;
    ctx->recorded = true;
    return SWARM_OK;
}

swarm_status swarm_capture_end(swarm_ctx* ctx, swarm_graph** out) {
    if (!ctx || !out) return SWARM_EINVAL;
    *out = nullptr;
    if (!ctx->capturing) SWARM_REJECT(ctx, "capture_end: not recording");
    ctx->capturing = false;
    hipGraph_t graph = nullptr;
    SWARM_HIP(ctx, hipStreamEndCapture(ctx->stream, &graph));
    hipGraphExec_t exec = nullptr;
    hipError_t e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
    if (e != hipSuccess) {
        (void)hipGraphDestroy(graph);
        snprintf(ctx->err, sizeof(ctx->err), "hipGraphInstantiate failed: %s", hipGetErrorString(e));
        return SWARM_EHIP;
    }
    swarm_graph* g = new (std::nothrow) swarm_graph();
    if (!g) { (void)hipGraphExecDestroy(exec); (void)hipGraphDestroy(graph); return SWARM_ENOMEM; }
    g->graph = graph;
    g->exec = exec;
    *out = g;
    return SWARM_OK;
}

swarm_status swarm_graph_launch(swarm_ctx* ctx, swarm_graph* graph) {
    if (!ctx || !graph) return SWARM_EINVAL;
    if (ctx->capturing) SWARM_REJECT(ctx, "graph_launch: not while recording");
    SWARM_HIP(ctx, hipGraphLaunch(graph->exec, ctx->stream));
    return SWARM_OK;
}

swarm_status swarm_graph_destroy(swarm_graph* graph) {
    if (!graph) return SWARM_EINVAL;
    if (graph->exec) (void)hipGraphExecDestroy(graph->exec);
    if (graph->graph) (void)hipGraphDestroy(graph->graph);
    delete graph;
    return SWARM_OK;
}

}  // extern "C"
