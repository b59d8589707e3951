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
#include <type_traits>

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
template <int LPR, int NCH, int UNROLL, bool PAGE, bool HM>
__global__ __launch_bounds__(256) void score_kernel(const u32x4* __restrict__ rows, const uint16_t* __restrict__ q,
                                                    float* __restrict__ out, int N, int H, int hshift, int G, int d, int CH,
                                                    const int32_t* __restrict__ row_ids, int M, uint32_t* __restrict__ dev_flags) {
    constexpr int RPW = 64 / LPR;
    constexpr int RPB = 4 * UNROLL * RPW;
    // Heads vary fastest over the workgroup id.  Workgroups are dealt to the eight XCDs round-robin, so with
    // eight heads all of a head's scores are produced, and stay cached, on the XCD whose L2 the workgroup that
    // selects from them (workgroup h of the next kernel) sits behind: its first read of the scores is an L2 hit
    // instead of a trip to memory (0.4 us per decode step, measured on one device against the head-slowest order).
    // (HM: H is a power of two, 2^hshift; otherwise the head is the grid's y as before -- a run-time choice with a
    // division in its other arm made the kernel's start 0.3 us slower.)
    const int b = blockIdx.z;
    const int h = HM ? (int)(blockIdx.x & (H - 1)) : (int)blockIdx.y;
    const int bx = HM ? (int)(blockIdx.x >> hshift) : (int)blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane % LPR, grp = lane / LPR;

    // With a row list (medoid index, Section 5.2 Tier 1) output row n is the score of entry row_ids[h][n];
    // an id outside [0,N) scores 0 and is flagged.
    const u32x4* base = rows + (size_t)h * N * CH;
    const int nout = row_ids ? M : N;
    const int32_t* ids = row_ids ? row_ids + (size_t)h * M : nullptr;
    float* o = out + ((size_t)b * H + h) * nout;
    bool chunk_ok[NCH];
#pragma unroll
    for (int m = 0; m < NCH; ++m) chunk_ok[m] = sub + m * LPR < CH;

    // The key rows first: their loads depend on nothing but the workgroup's position, and they are the long trip
    // (memory).  The query is fetched and folded into the weights while they are in flight; loading the query first
    // put one cache round trip in front of every workgroup's first memory request.
    // Every lane loads from a valid address (row and chunk clamped) and what it must not use is zeroed afterwards:
    // no divergent branch sits between the loads, so all of them are in flight together.
    const int row0 = bx * RPB + wave * UNROLL * RPW + grp;
    int src[UNROLL];
    bool use[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        src[u] = min(row0 + u * RPW, nout - 1);
        use[u] = true;
    }
    if (ids) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) src[u] = ids[src[u]];
        bool bad = false;
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            use[u] = (uint32_t)src[u] < (uint32_t)N;
            bad |= !use[u] && row0 + u * RPW < nout;
            src[u] = use[u] ? src[u] : 0;
        }
        if (bad) atomicOr(dev_flags, SWARM_DEV_BAD_ENTRY);
    }
    u32x4 x[UNROLL][NCH];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u)
#pragma unroll
        for (int m = 0; m < NCH; ++m)
            x[u][m] = __builtin_nontemporal_load(base + (size_t)src[u] * CH + min(sub + m * LPR, CH - 1));
#pragma unroll
    for (int u = 0; u < UNROLL; ++u)
#pragma unroll
        for (int m = 0; m < NCH; ++m)
            if (!(use[u] && chunk_ok[m])) x[u][m] = u32x4{0, 0, 0, 0};

    const uint16_t* qbh = q + ((size_t)b * H + h) * (size_t)G * d;
    float w[NCH][8];
#pragma unroll
    for (int m = 0; m < NCH; ++m) {
        if (chunk_ok[m]) load_weights<PAGE>(qbh, G, d, sub + m * LPR, w[m]);
        else {
#pragma unroll
            for (int e = 0; e < 8; ++e) w[m][e] = 0.f;
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
        if (sub < UNROLL && n < nout) o[n] = v;
    } else {
        if (sub == 0) {
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const int n = row0 + u * RPW;
                if (n < nout) o[n] = p[u];
            }
        }
    }
}


// Lean form of the sweep for the shapes the decode path runs on: one query head per KV head (G = 1), a row of
// exactly LPR chunks, a power-of-two number of heads (heads fastest over the workgroup id, as above), no row list.
// The sweep moves 16 KiB per workgroup and every one of the 2048 workgroups of a 33.5 MB launch runs its code once:
// measured on one device, the launch takes 7.3 us with 430 instructions per wave, 6.7 us with 254 and 6.5 us with
// 125 -- what a wave executes around its four loads is time the memory system waits for its next request.  Hence:
// compile-time row length, one address per wave with literal offsets for the other rows, and a reduction that
// halves the values a lane carries while it halves the lanes (two exchange steps bring a lane's four partial sums
// down to one, which then needs one add per remaining lane stride: 6 exchanges instead of 20).
template <int LPR, bool PAGE>
__global__ __launch_bounds__(256) void score_lean_kernel(const u32x4* __restrict__ rows, const uint16_t* __restrict__ q,
                                                         float* __restrict__ out, int N, int H, int hshift) {
    constexpr int RPW = 64 / LPR, UNROLL = 4, RPB = 4 * UNROLL * RPW, CH = LPR;
    constexpr int D = PAGE ? CH * 4 : CH * 8;                 // head dimension
    static_assert(LPR >= 8 && LPR <= 32, "");
    const int b = blockIdx.z;
    const int h = (int)(blockIdx.x & (H - 1)), bx = (int)(blockIdx.x >> hshift);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane % LPR, grp = lane / LPR;
    const int row0 = bx * RPB + wave * UNROLL * RPW + grp;
    const u32x4* base = rows + (size_t)h * N * CH;

    u32x4 x[UNROLL];
    if ((bx + 1) * RPB <= N) {                                // the whole workgroup inside the head: one address, literal offsets
        const u32x4* p0 = base + (size_t)row0 * CH + sub;
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) x[u] = __builtin_nontemporal_load(p0 + u * RPW * CH);
    } else {                                                  // the head's last workgroup: rows clamped, stores masked below
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) x[u] = __builtin_nontemporal_load(base + (size_t)min(row0 + u * RPW, N - 1) * CH + sub);
    }

    // weights of this lane's chunk, fetched while the rows are in flight
    float w[8];
    {
        const bool max_half = PAGE && sub >= LPR / 2;
        const int c0 = (PAGE ? sub % (LPR / 2) : sub) * 8;
        const u32x4 v = *reinterpret_cast<const u32x4*>(q + ((size_t)b * H + h) * D + c0);
        const float f[8] = {bf16_lo(v.x), bf16_hi(v.x), bf16_lo(v.y), bf16_hi(v.y), bf16_lo(v.z), bf16_hi(v.z), bf16_lo(v.w), bf16_hi(v.w)};
#pragma unroll
        for (int e = 0; e < 8; ++e) w[e] = PAGE ? (max_half ? fmaxf(f[e], 0.f) : fminf(f[e], 0.f)) : f[e];
    }
    float p[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) p[u] = dot8(x[u], w);

    // lanes exchange with the partner one lane away and keep rows {0,1} (even lane) or {2,3} (odd lane), then two lanes
    // away and keep one row; the lanes of a row's group that agree in their two low bits then add up
    auto dpp = [](float v, auto ctrl) __attribute__((always_inline)) {
        return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), decltype(ctrl)::value, 0xF, 0xF, true));
    };
    const bool b0 = lane & 1, b1 = lane & 2;
    float k0 = b0 ? p[2] : p[0], k1 = b0 ? p[3] : p[1];
    const float s0 = b0 ? p[0] : p[2], s1 = b0 ? p[1] : p[3];
    k0 += dpp(s0, std::integral_constant<int, 0xB1>{});       // quad_perm [1,0,3,2]
    k1 += dpp(s1, std::integral_constant<int, 0xB1>{});
    float v = b1 ? k1 : k0;
    const float sv = b1 ? k0 : k1;
    v += dpp(sv, std::integral_constant<int, 0x4E>{});        // quad_perm [2,3,0,1]
    if (LPR == 8) {
        v += __shfl_xor(v, 4, 64);                            // a rotation inside 16 lanes would reach into the neighbouring group of 8
    } else {
        v += dpp(v, std::integral_constant<int, 0x124>{});    // row_ror:4  (rotation inside a row of 16 lanes)
        v += dpp(v, std::integral_constant<int, 0x128>{});    // row_ror:8
    }
    if (LPR >= 32) v += __shfl_xor(v, 16, 64);
    // lane (b0, b1) of a group now holds row 2 b0 + b1 of its group's four rows
    const int n = row0 + (2 * (int)b0 + (int)(b1 ? 1 : 0)) * RPW;
    if (sub < UNROLL && n < N) out[((size_t)b * H + h) * N + n] = v;
}

template <int LPR, int NCH, bool PAGE>
void launch_one(hipStream_t st, const swarm_keys* keys, const void* q, int B, float* scores, int CH, const int32_t* row_ids,
                int M, uint32_t* dev_flags) {
    constexpr int UNROLL = (NCH == 2 || LPR >= 16) ? 4 : 8;
    constexpr int RPB = 4 * UNROLL * (64 / LPR);
    const int gxn = ((row_ids ? M : keys->N) + RPB - 1) / RPB;      // one row group per workgroup
    if ((keys->H & (keys->H - 1)) == 0) {                   // power of two: heads fastest over the workgroup id
        hipLaunchKernelGGL((score_kernel<LPR, NCH, UNROLL, PAGE, true>), dim3(gxn * keys->H, 1, B), dim3(256), 0, st,
                           static_cast<const u32x4*>(keys->data), static_cast<const uint16_t*>(q), scores, keys->N, keys->H,
                           __builtin_ctz(keys->H), keys->G, keys->d, CH, row_ids, M, dev_flags);
    } else {
        hipLaunchKernelGGL((score_kernel<LPR, NCH, UNROLL, PAGE, false>), dim3(gxn, keys->H, B), dim3(256), 0, st,
                           static_cast<const u32x4*>(keys->data), static_cast<const uint16_t*>(q), scores, keys->N, keys->H,
                           0, keys->G, keys->d, CH, row_ids, M, dev_flags);
    }
}

template <int LPR, bool PAGE>
void launch_lean(hipStream_t st, const swarm_keys* keys, const void* q, int B, float* scores) {
    constexpr int RPB = 4 * 4 * (64 / LPR);
    const int gxn = (keys->N + RPB - 1) / RPB;
    hipLaunchKernelGGL((score_lean_kernel<LPR, PAGE>), dim3(gxn * keys->H, 1, B), dim3(256), 0, st, static_cast<const u32x4*>(keys->data),
                       static_cast<const uint16_t*>(q), scores, keys->N, keys->H, __builtin_ctz(keys->H));
}

template <bool PAGE>
void dispatch(hipStream_t st, const swarm_keys* keys, const void* q, int B, float* scores, int CH, const int32_t* row_ids, int M,
              uint32_t* dev_flags) {
    if (!row_ids && keys->G == 1 && (keys->H & (keys->H - 1)) == 0) {      // the decode path's shapes: the lean kernel
        if (CH == 32) return launch_lean<32, PAGE>(st, keys, q, B, scores);
        if (CH == 16) return launch_lean<16, PAGE>(st, keys, q, B, scores);
        if (CH == 8) return launch_lean<8, PAGE>(st, keys, q, B, scores);
    }
    if (CH > 64) return launch_one<64, 2, PAGE>(st, keys, q, B, scores, CH, row_ids, M, dev_flags);
    if (CH > 32) return launch_one<64, 1, PAGE>(st, keys, q, B, scores, CH, row_ids, M, dev_flags);
    if (CH > 16) return launch_one<32, 1, PAGE>(st, keys, q, B, scores, CH, row_ids, M, dev_flags);
    if (CH > 8) return launch_one<16, 1, PAGE>(st, keys, q, B, scores, CH, row_ids, M, dev_flags);
    if (CH > 4) return launch_one<8, 1, PAGE>(st, keys, q, B, scores, CH, row_ids, M, dev_flags);
    if (CH > 2) return launch_one<4, 1, PAGE>(st, keys, q, B, scores, CH, row_ids, M, dev_flags);
    if (CH > 1) return launch_one<2, 1, PAGE>(st, keys, q, B, scores, CH, row_ids, M, dev_flags);
    return launch_one<1, 1, PAGE>(st, keys, q, B, scores, CH, row_ids, M, dev_flags);
}


// ---- many streams per call: the sweep becomes a small GEMM on the bf16 matrix cores -------------
//
// s[b][n] = sum_g sum_c w_g[b][c] * row[n][c], w_g the weights of query head g of stream b: the query itself for
// token keys, [min(q,0), max(q,0)] for page summaries.  Clamping a bf16 against zero leaves a bf16, so every
// weight is exact and the G query heads of a group are G matrix-core products into one fp32 accumulator: no
// folded fp32 weights, no split into a high and a low part, no separate launch to prepare them.
// A workgroup owns 128 entries (32 per wave, read from memory once, straight into the A fragments) and one tile
// of 32 streams; the weights of that tile are staged in LDS, clamped on the way (both clamped versions of a page
// query are stored, the lane half picks its own).  The contraction index is free to be visited in any order as
// long as both operands agree: lane half 0 walks the first half of the row, lane half 1 the second half, 8 values
// per k-step, so every lane reads one contiguous run of its row -- and for page rows the first half is the min
// summary, the second the max summary, so both halves of a k-step use the same 8 query channels.

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int SB_GT = 4;        // query heads of a group staged per pass

// The negative ones of two packed bf16 values (min(q,0)); the other version, max(q,0), is what is left of the pair.
// A NaN goes where its sign bit says, so a NaN query makes its scores NaN.
__device__ __forceinline__ uint32_t negative_halves(uint32_t v) {
    const uint32_t sign = (v >> 15) & 0x00010001u;
    return v & ((sign << 16) - sign);                            // mask: 0xffff in every half whose sign bit is set
}

// grid (ceil(N / 128), H, ceil(B / 32)); 4 waves, wave w scores entries [128 x + 32 w, +32) for streams [32 z, +32).
// KSTEPS = L / 16 k-steps, each consuming 8 values from each half of the row.  LDS: [SB_GT][NVER][32][WROW] chunks.
template <int KSTEPS, bool PAGE>
__global__ __launch_bounds__(256) void score_batched_kernel(const u32x4* __restrict__ rows, const u32x4* __restrict__ q,
                                                            float* __restrict__ out, int N, int H, int B, int G) {
    constexpr int CH = KSTEPS * 2;                         // 16-byte chunks per key row
    constexpr int CHQ = PAGE ? KSTEPS : KSTEPS * 2;        // 16-byte chunks per query vector (d / 8)
    constexpr int WROW = CHQ + 1;                          // padded: the 16 lanes an LDS read serves together fall into 16 bank groups
    constexpr int NVER = PAGE ? 2 : 1;
    extern __shared__ __attribute__((aligned(16))) u32x4 wt[];
    const int h = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r32 = lane & 31, hf = lane >> 5;
    const int n0 = blockIdx.x * 128 + wave * 32;
    const int b0 = blockIdx.z * 32;
    const int n = min(n0 + r32, N - 1);                                     // clamped; stores are masked
    const u32x4* arow = rows + ((size_t)h * N + n) * CH + hf * KSTEPS;

    // The first pass's query chunks are requested before the key rows: they come from the cache and are clamped and
    // parked in LDS while the rows are still on their way from memory.
    constexpr int NPRE = SB_GT * 32 * CHQ / 256;          // staged chunks per thread and pass
    auto fetch = [&](int g0, int gn, u32x4 (&qv)[NPRE]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NPRE; ++i) {
            const int u = threadIdx.x + i * 256;
            const int c = u % CHQ, sb = (u / CHQ) & 31, g = min(u / (CHQ * 32), gn - 1);
            const int b = min(b0 + sb, B - 1);
            qv[i] = q[(((size_t)b * H + h) * G + g0 + g) * CHQ + c];
        }
    };
    auto park = [&](int gn, const u32x4 (&qv)[NPRE]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NPRE; ++i) {
            const int u = threadIdx.x + i * 256;
            const int c = u % CHQ, sb = (u / CHQ) & 31, g = u / (CHQ * 32);
            if (g < gn) {
                u32x4* dst = wt + ((size_t)g * NVER * 32 + sb) * WROW + c;
                const u32x4 v = qv[i];
                if (PAGE) {
                    const u32x4 neg = {negative_halves(v.x), negative_halves(v.y), negative_halves(v.z), negative_halves(v.w)};
                    dst[0] = neg;                          // min(q, 0): weights of the min half
                    dst[32 * WROW] = v ^ neg;              // max(q, 0): weights of the max half
                } else {
                    dst[0] = v;
                }
            }
        }
    };
    u32x4 qv[NPRE];
    fetch(0, min(SB_GT, G), qv);
    u32x4 a[KSTEPS];
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) a[s] = arow[s];      // cached loads: a 128-byte line serves eight consecutive k-steps of a lane

    f32x16 acc, acc1;                                      // two chains of dependent MFMAs: the wave is alone on its SIMD
#pragma unroll
    for (int r = 0; r < 16; ++r) { acc[r] = 0.f; acc1[r] = 0.f; }

    for (int g0 = 0; g0 < G; g0 += SB_GT) {
        const int gn = min(SB_GT, G - g0);
        if (g0) {
            __syncthreads();                               // the previous pass's fragments have been read
            fetch(g0, gn, qv);
        }
        park(gn, qv);
        __syncthreads();
        // The weight fragments of query head g + 1 are read from LDS while head g's MFMAs run (two register sets): read
        // one k-step ahead, every pair of MFMAs waited for an LDS round trip of its own, 64 of them per wave.  What is left
        // of this phase is LDS bandwidth: every wave reads all of the tile's weights (1 KiB per MFMA and SIMD).
        u32x4 wb[2][KSTEPS];
        auto read_frags = [&](int set, int g) __attribute__((always_inline)) {
            const u32x4* wf = wt + ((size_t)(g * NVER + (PAGE ? hf : 0)) * 32 + r32) * WROW + (PAGE ? 0 : hf * KSTEPS);
#pragma unroll
            for (int s = 0; s < KSTEPS; ++s) wb[set][s] = wf[s];
        };
        read_frags(0, 0);
#pragma unroll
        for (int g = 0; g < SB_GT; ++g) {
            if (g < gn) {
                if (g + 1 < SB_GT && g + 1 < gn) read_frags((g + 1) & 1, g + 1);
#pragma unroll
                for (int s = 0; s < KSTEPS; s += 2) {
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[s]), __builtin_bit_cast(bf16x8, wb[g & 1][s]), acc, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[s + 1]), __builtin_bit_cast(bf16x8, wb[g & 1][s + 1]), acc1, 0, 0, 0);
                }
            }
        }
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] += acc1[r];
    // result tile: lane l, register r -> stream b0 + l%32, entry n0 + 8*(r/4) + 4*(l/32) + r%4
    const int b = b0 + r32;
    if (b < B) {
        float* o = out + ((size_t)b * H + h) * N;
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
            const int nn = n0 + rq * 8 + hf * 4;
            if (nn + 3 < N && ((reinterpret_cast<uintptr_t>(o + nn) & 15) == 0)) {
                *reinterpret_cast<float4*>(o + nn) = make_float4(acc[rq * 4], acc[rq * 4 + 1], acc[rq * 4 + 2], acc[rq * 4 + 3]);
            } else {
#pragma unroll
                for (int rr = 0; rr < 4; ++rr)
                    if (nn + rr < N) o[nn + rr] = acc[rq * 4 + rr];
            }
        }
    }
}

template <int KSTEPS, bool PAGE>
swarm_status launch_batched(swarm_ctx* ctx, const swarm_keys* keys, const void* q, int B, float* scores) {
    constexpr int CHQ = PAGE ? KSTEPS : KSTEPS * 2;
    constexpr size_t LDS = (size_t)SB_GT * (PAGE ? 2 : 1) * 32 * (CHQ + 1) * 16;
    if (LDS > 64 * 1024 && !ctx->batched_lds_opt_in) {     // per context: the attribute belongs to the device the context is bound to
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&score_batched_kernel<KSTEPS, PAGE>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS);
        if (e != hipSuccess) {
            snprintf(ctx->err, sizeof(ctx->err), "score: cannot opt in to %zu bytes of LDS: %s", LDS, hipGetErrorString(e));
            return SWARM_EHIP;
        }
        ctx->batched_lds_opt_in = true;
    }
    dim3 grid((keys->N + 127) / 128, keys->H, (B + 31) / 32);
    hipLaunchKernelGGL((score_batched_kernel<KSTEPS, PAGE>), grid, dim3(256), LDS, ctx->stream, static_cast<const u32x4*>(keys->data),
                       static_cast<const u32x4*>(q), scores, keys->N, keys->H, B, keys->G);
    return swarm_check_launch(ctx, "score_batched_kernel");
}

}  // namespace

static bool score_is_batched(const swarm_keys* keys, int B, bool listed) {
    const int L = keys->kind == SWARM_KEYS_PAGE_MINMAX ? 2 * keys->d : keys->d;
    return !listed && B >= SWARM_BATCHED_MIN_STREAMS && (L == 128 || L == 256) && keys->H <= 65535;
}

swarm_status launch_score(swarm_ctx* ctx, const swarm_keys* keys, const void* q, int B, float* scores, const int32_t* row_ids,
                          int M) {
    if (((int64_t)(row_ids ? M : keys->N) / 16 + 1) * keys->H > 0x7fffffffll) {       // workgroups along x: at least 16 rows each
        snprintf(ctx->err, sizeof(ctx->err), "score: N=%d x H=%d is more than one launch can cover", keys->N, keys->H);
        return SWARM_EINVAL;
    }
    if (B > 65535 || keys->H > 65535) {
        snprintf(ctx->err, sizeof(ctx->err), "score: B=%d and H=%d must each be below 65536", B, keys->H);
        return SWARM_EINVAL;
    }
    const bool page = keys->kind == SWARM_KEYS_PAGE_MINMAX;
    const int L = page ? 2 * keys->d : keys->d;
    const int CH = L / 8;
    // many streams: matrix-core path (row lengths of 128 and 256 values, i.e. d = 128 or page rows of d = 64 / 128)
    // many streams: matrix-core path (row lengths of 128 and 256 values, i.e. d = 128 or page rows of d = 64 / 128)
    if (score_is_batched(keys, B, row_ids != nullptr)) {
        if (page) return L == 256 ? launch_batched<16, true>(ctx, keys, q, B, scores) : launch_batched<8, true>(ctx, keys, q, B, scores);
        return L == 256 ? launch_batched<16, false>(ctx, keys, q, B, scores) : launch_batched<8, false>(ctx, keys, q, B, scores);
    }
    if (page) dispatch<true>(ctx->stream, keys, q, B, scores, CH, row_ids, M, ctx->dev_flags);
    else dispatch<false>(ctx->stream, keys, q, B, scores, CH, row_ids, M, ctx->dev_flags);
    return swarm_check_launch(ctx, "score_kernel");
}
