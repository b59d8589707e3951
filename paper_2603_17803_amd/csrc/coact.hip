// Trace scatter and co-activation accumulation (Section 5.1, Step 1): C[i][j] = number of trace
// rows in which entries i and j are both activated, i.e. C = A^T A for the binary trace A.
//
// The trace is kept entry-major, At[h][n][t] (int8 0/1), so that both operands of the product are
// rows of the same matrix with the contraction index t contiguous: C[i][j] = <At[i], At[j]>.
// The product runs on the int8 matrix cores (v_mfma_i32_32x32x32_i8) with exact int32
// accumulation.  C is symmetric, so only tiles on or above the diagonal are computed and each
// off-diagonal tile is stored twice (once transposed).
#include "common.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

__global__ void fill_zero_kernel(uint4* __restrict__ p, size_t n16) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) p[i] = make_uint4(0, 0, 0, 0);
}

// One thread per selected entry: At[h][e][row] = 1.
__global__ void trace_scatter_kernel(const int32_t* __restrict__ idx, int64_t total, int H, int k, int N, int Npad,
                                     int64_t Tpad, int8_t* __restrict__ At, uint32_t* __restrict__ dev_flags) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int64_t rh = i / k;
    const int64_t row = rh / H;
    const int h = (int)(rh % H);
    const int32_t e = idx[i];
    if (e < 0 || e >= N) { atomicOr(dev_flags, SWARM_DEV_BAD_ENTRY); return; }
    At[((size_t)h * Npad + e) * Tpad + row] = 1;
}

// Optional validation: flags a repeated entry inside one (row, head) selection.
__global__ void check_distinct_kernel(const int32_t* __restrict__ idx, int k, uint32_t* __restrict__ dev_flags) {
    const int32_t* sel = idx + (size_t)blockIdx.x * k;
    bool dup = false;
    for (int a = threadIdx.x; a < k; a += blockDim.x) {
        const int32_t e = sel[a];
        for (int b = 0; b < a; ++b) dup |= (sel[b] == e);
    }
    if (dup) atomicOr(dev_flags, SWARM_DEV_DUP_ENTRY);
}

__device__ __forceinline__ int32_t decayed(int32_t old, uint32_t decay_q16) {
    return (int32_t)(((int64_t)old * (int64_t)decay_q16 + 32768) >> 16);
}

// MODE 0: C = acc.  MODE 1: C += acc.  MODE 2: C = decayed(C) + acc.
template <int MODE>
__device__ __forceinline__ void store_c(int32_t* p, int32_t acc, uint32_t decay_q16) {
    if (MODE == 0) *p = acc;
    else if (MODE == 1) *p += acc;
    else *p = decayed(*p, decay_q16) + acc;
}

constexpr int TILE = 128;      // C tile edge per workgroup
constexpr int KC = 64;         // contraction bytes staged per iteration
constexpr int LDS_ROW = KC + 16;   // padded LDS row (bytes)

// 256 threads = 4 waves in a 2x2 arrangement, each wave owns a 64x64 corner = 2x2 MFMA tiles.
template <int MODE>
__global__ __launch_bounds__(256) void coact_syrk_kernel(const int8_t* __restrict__ At, int N, int Npad, int64_t Tpad,
                                                         int32_t* __restrict__ C, uint32_t decay_q16) {
    const int ti = blockIdx.y, tj = blockIdx.x, h = blockIdx.z;
    if (tj < ti) return;                                       // lower triangle comes from the mirror store
    __shared__ __attribute__((aligned(16))) int8_t lds_a[TILE * LDS_ROW];
    __shared__ __attribute__((aligned(16))) int8_t lds_b[TILE * LDS_ROW];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wy = wave >> 1, wx = wave & 1;
    const int8_t* a_rows = At + ((size_t)h * Npad + (size_t)ti * TILE) * Tpad;
    const int8_t* b_rows = At + ((size_t)h * Npad + (size_t)tj * TILE) * Tpad;

    // staging: thread t copies 16 bytes of row t/4 (and t/4 + 64), byte column (t%4)*16
    const int srow = tid >> 2, scol = (tid & 3) * 16;

    v16i acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    const int frow = lane & 31, fk = (lane >> 5) * 16;         // MFMA operand fragment: row, byte offset in a 32-byte k-step
    for (int64_t k0 = 0; k0 < Tpad; k0 += KC) {
        const v4i a0 = *reinterpret_cast<const v4i*>(a_rows + (size_t)srow * Tpad + k0 + scol);
        const v4i a1 = *reinterpret_cast<const v4i*>(a_rows + (size_t)(srow + 64) * Tpad + k0 + scol);
        const v4i b0 = *reinterpret_cast<const v4i*>(b_rows + (size_t)srow * Tpad + k0 + scol);
        const v4i b1 = *reinterpret_cast<const v4i*>(b_rows + (size_t)(srow + 64) * Tpad + k0 + scol);
        __syncthreads();                                       // previous iteration's reads are done
        *reinterpret_cast<v4i*>(lds_a + srow * LDS_ROW + scol) = a0;
        *reinterpret_cast<v4i*>(lds_a + (srow + 64) * LDS_ROW + scol) = a1;
        *reinterpret_cast<v4i*>(lds_b + srow * LDS_ROW + scol) = b0;
        *reinterpret_cast<v4i*>(lds_b + (srow + 64) * LDS_ROW + scol) = b1;
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < KC; ks += 32) {
            v4i fa[2], fb[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                fa[i] = *reinterpret_cast<const v4i*>(lds_a + (wy * 64 + i * 32 + frow) * LDS_ROW + ks + fk);
                fb[i] = *reinterpret_cast<const v4i*>(lds_b + (wx * 64 + i * 32 + frow) * LDS_ROW + ks + fk);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    }

    // 32x32 result layout: lane l, register r -> column l%32, row 8*(r/4) + 4*(l/32) + r%4
    int32_t* Ch = C + (size_t)h * N * N;
    const int col_in = lane & 31, row_in = (lane >> 5) * 4;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int gi = ti * TILE + wy * 64 + i * 32 + (r >> 2) * 8 + row_in + (r & 3);
                const int gj = tj * TILE + wx * 64 + j * 32 + col_in;
                if (gi < N && gj < N) {
                    const int32_t v = acc[i][j][r];
                    store_c<MODE>(Ch + (size_t)gi * N + gj, v, decay_q16);
                    if (tj != ti) store_c<MODE>(Ch + (size_t)gj * N + gi, v, decay_q16);
                }
            }
}

}  // namespace

swarm_status launch_trace_scatter(swarm_ctx* ctx, const int32_t* idx, int64_t rows, int H, int k, int N, int Npad,
                                  int64_t Tpad, uint32_t flags) {
    const size_t n16 = (size_t)H * Npad * Tpad / 16;
    const unsigned fill_blocks = (unsigned)((n16 + 255) / 256 < 16384 ? (n16 + 255) / 256 : 16384);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(fill_blocks), dim3(256), 0, ctx->stream,
                       reinterpret_cast<uint4*>(ctx->trace), n16);
    swarm_status st = swarm_check_launch(ctx, "fill_zero_kernel");
    if (st != SWARM_OK) return st;
    if (flags & SWARM_CHECK_IDX) {
        hipLaunchKernelGGL(check_distinct_kernel, dim3((unsigned)(rows * H)), dim3(256), 0, ctx->stream, idx, k,
                           ctx->dev_flags);
        st = swarm_check_launch(ctx, "check_distinct_kernel");
        if (st != SWARM_OK) return st;
    }
    const int64_t total = rows * H * k;
    hipLaunchKernelGGL(trace_scatter_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, ctx->stream, idx, total,
                       H, k, N, Npad, Tpad, ctx->trace, ctx->dev_flags);
    return swarm_check_launch(ctx, "trace_scatter_kernel");
}

swarm_status launch_coact_syrk(swarm_ctx* ctx, int H, int N, int Npad, int64_t Tpad, int32_t* C, uint32_t decay_q16) {
    const int nt = Npad / TILE;
    if (nt > 65535 || H > 65535) {
        snprintf(ctx->err, sizeof(ctx->err), "coact: N=%d or H=%d too large for the launch grid", N, H);
        return SWARM_EINVAL;
    }
    dim3 grid(nt, nt, H), block(256);
    if (decay_q16 == 0u)
        hipLaunchKernelGGL(coact_syrk_kernel<0>, grid, block, 0, ctx->stream, ctx->trace, N, Npad, Tpad, C, decay_q16);
    else if (decay_q16 == 65536u)
        hipLaunchKernelGGL(coact_syrk_kernel<1>, grid, block, 0, ctx->stream, ctx->trace, N, Npad, Tpad, C, decay_q16);
    else
        hipLaunchKernelGGL(coact_syrk_kernel<2>, grid, block, 0, ctx->stream, ctx->trace, N, Npad, Tpad, C, decay_q16);
    return swarm_check_launch(ctx, "coact_syrk_kernel");
}
