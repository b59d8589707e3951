// Scoring step (Section 2.3): relevance score of every KV entry against the query.
//
// Both key kinds reduce to one streamed dot product per entry.  A token key is a row of d bf16
// values and s = sum_c q_c * K_c.  A page summary is a row of 2d values (min half, then max
// half) and max(q*mn, q*mx) equals min(q,0)*mn + max(q,0)*mx because mn <= mx, so
// s = sum_c w_c * row_c with w = [min(q,0), max(q,0)].  With grouped-query attention the
// G query heads add, and since the form is linear in w they are folded into w up front.
//
// The sweep is bound by HBM bandwidth: each lane issues UNROLL independent 16-byte loads, a
// group of LPR lanes covers one row, a wave covers 64/LPR consecutive rows per load (1 KiB
// contiguous), and the per-row partial sums are combined with a lane butterfly.
#include "common.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

__device__ __forceinline__ float dot8(const u32x4& x, const float (&w)[8]) {
    float s = bf16_lo(x.x) * w[0];
    s = fmaf(bf16_hi(x.x), w[1], s);
    s = fmaf(bf16_lo(x.y), w[2], s);
    s = fmaf(bf16_hi(x.y), w[3], s);
    s = fmaf(bf16_lo(x.z), w[4], s);
    s = fmaf(bf16_hi(x.z), w[5], s);
    s = fmaf(bf16_lo(x.w), w[6], s);
    s = fmaf(bf16_hi(x.w), w[7], s);
    return s;
}

// Query weights of one 8-channel chunk of the row, summed over the G heads of the group.
template <bool PAGE>
__device__ __forceinline__ void load_weights(const uint16_t* __restrict__ qbh, int G, int d, int chunk, float (&w)[8]) {
    int c0 = chunk * 8;
    bool max_half = false;
    if (PAGE && c0 >= d) { c0 -= d; max_half = true; }
#pragma unroll
    for (int e = 0; e < 8; ++e) w[e] = 0.f;
    for (int g = 0; g < G; ++g) {
        const u32x4 v = *reinterpret_cast<const u32x4*>(qbh + (size_t)g * d + c0);
        float f[8] = {bf16_lo(v.x), bf16_hi(v.x), bf16_lo(v.y), bf16_hi(v.y),
                      bf16_lo(v.z), bf16_hi(v.z), bf16_lo(v.w), bf16_hi(v.w)};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float x = f[e];
            if (PAGE) x = max_half ? fmaxf(x, 0.f) : fminf(x, 0.f);
            w[e] += x;
        }
    }
}

// LPR lanes per row (power of two), NCH chunks per lane (row longer than 64 chunks), UNROLL
// rows in flight per lane.  CH = 16-byte chunks per row.
template <int LPR, int NCH, int UNROLL, bool PAGE>
__global__ __launch_bounds__(256) void score_kernel(const u32x4* __restrict__ rows, const uint16_t* __restrict__ q,
                                                    float* __restrict__ out, int N, int H, int G, int d, int CH, int iters) {
    constexpr int RPW = 64 / LPR;
    constexpr int RPB = 4 * UNROLL * RPW;
    const int h = blockIdx.y, b = blockIdx.z;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane % LPR, grp = lane / LPR;

    const uint16_t* qbh = q + ((size_t)b * H + h) * (size_t)G * d;
    float w[NCH][8];
    bool chunk_ok[NCH];
#pragma unroll
    for (int m = 0; m < NCH; ++m) {
        const int chunk = sub + m * LPR;
        chunk_ok[m] = chunk < CH;
        if (chunk_ok[m]) load_weights<PAGE>(qbh, G, d, chunk, w[m]);
        else {
#pragma unroll
            for (int e = 0; e < 8; ++e) w[m][e] = 0.f;
        }
    }

    const u32x4* base = rows + (size_t)h * N * CH;
    float* o = out + ((size_t)b * H + h) * N;
    // `iters` row groups per workgroup, a grid width apart: fewer, longer-lived workgroups measured
    // a few percent faster on long sweeps
#pragma unroll 1
    for (int it = 0; it < iters; ++it) {
    const int row0 = (blockIdx.x + it * gridDim.x) * RPB + wave * UNROLL * RPW + grp;
    u32x4 x[UNROLL][NCH];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int n = row0 + u * RPW;
#pragma unroll
        for (int m = 0; m < NCH; ++m) {
            if (n < N && chunk_ok[m]) x[u][m] = __builtin_nontemporal_load(base + (size_t)n * CH + sub + m * LPR);
            else x[u][m] = u32x4{0, 0, 0, 0};
        }
    }
    float p[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        float s = 0.f;
#pragma unroll
        for (int m = 0; m < NCH; ++m) s += dot8(x[u][m], w[m]);
        p[u] = s;
    }
#pragma unroll
    for (int off = LPR / 2; off >= 1; off >>= 1) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) p[u] += __shfl_xor(p[u], off, 64);
    }
    if constexpr (LPR >= UNROLL) {
        // lane `sub` of each group stores row u = sub: 64/LPR * UNROLL consecutive floats per wave
        float v = p[0];
#pragma unroll
        for (int u = 1; u < UNROLL; ++u) v = (sub == u) ? p[u] : v;
        const int n = row0 + sub * RPW;
        if (sub < UNROLL && n < N) o[n] = v;
    } else {
        if (sub == 0) {
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const int n = row0 + u * RPW;
                if (n < N) o[n] = p[u];
            }
        }
    }
    }
}


template <int LPR, int NCH, bool PAGE>
void launch_one(hipStream_t st, const swarm_keys* keys, const void* q, int B, float* scores, int CH) {
    constexpr int UNROLL = (NCH == 2 || LPR >= 16) ? 4 : 8;
    constexpr int RPB = 4 * UNROLL * (64 / LPR);
    const int groups = (keys->N + RPB - 1) / RPB;
    const int iters = ((long)groups * keys->H * B >= 2048) ? 2 : 1;
    dim3 grid((groups + iters - 1) / iters, keys->H, B);
    hipLaunchKernelGGL((score_kernel<LPR, NCH, UNROLL, PAGE>), grid, dim3(256), 0, st,
                       static_cast<const u32x4*>(keys->data), static_cast<const uint16_t*>(q), scores, keys->N, keys->H,
                       keys->G, keys->d, CH, iters);
}

template <bool PAGE>
void dispatch(hipStream_t st, const swarm_keys* keys, const void* q, int B, float* scores, int CH) {
    if (CH > 64) return launch_one<64, 2, PAGE>(st, keys, q, B, scores, CH);
    if (CH > 32) return launch_one<64, 1, PAGE>(st, keys, q, B, scores, CH);
    if (CH > 16) return launch_one<32, 1, PAGE>(st, keys, q, B, scores, CH);
    if (CH > 8) return launch_one<16, 1, PAGE>(st, keys, q, B, scores, CH);
    if (CH > 4) return launch_one<8, 1, PAGE>(st, keys, q, B, scores, CH);
    if (CH > 2) return launch_one<4, 1, PAGE>(st, keys, q, B, scores, CH);
    if (CH > 1) return launch_one<2, 1, PAGE>(st, keys, q, B, scores, CH);
    return launch_one<1, 1, PAGE>(st, keys, q, B, scores, CH);
}

}  // namespace

swarm_status launch_score(swarm_ctx* ctx, const swarm_keys* keys, const void* q, int B, float* scores) {
    if (B > 65535 || keys->H > 65535) {
        snprintf(ctx->err, sizeof(ctx->err), "score: B=%d and H=%d must each be below 65536", B, keys->H);
        return SWARM_EINVAL;
    }
    const bool page = keys->kind == SWARM_KEYS_PAGE_MINMAX;
    const int CH = (page ? 2 * keys->d : keys->d) / 8;
    if (page) dispatch<true>(ctx->stream, keys, q, B, scores, CH);
    else dispatch<false>(ctx->stream, keys, q, B, scores, CH);
    return swarm_check_launch(ctx, "score_kernel");
}
