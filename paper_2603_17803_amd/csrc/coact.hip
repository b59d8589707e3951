// Trace scatter and co-activation accumulation (Section 5.1, Step 1): C[i][j] = number of trace
// rows in which entries i and j are both activated, i.e. C = A^T A for the binary trace A.
//
// The trace is kept entry-major, At[h][n][t] (int8 0/1), so that both operands of the product are
// rows of the same matrix with the contraction index t contiguous: C[i][j] = <At[i], At[j]>.
// The product runs on the int8 matrix cores (v_mfma_i32_32x32x32_i8) with exact int32
// accumulation.  C is symmetric, so only tiles on or above the diagonal are computed and each
// off-diagonal tile is stored twice (once transposed).
#include <stdlib.h>

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

// floor((old * decay_q16 + 2^15) / 2^16) with a 64-bit intermediate (one 64-bit multiply-add and a
// funnel shift; decay_q16 <= 65536, so the result fits int32).
__device__ __forceinline__ int32_t decayed(int32_t old, uint32_t decay_q16) {
    return (int32_t)(((int64_t)old * (int64_t)decay_q16 + 32768) >> 16);
}

// MODE 0: C = acc.  MODE 1: C += acc.  MODE 2: C = decayed(C) + acc.
constexpr int TILE = 256;          // C tile edge per workgroup
constexpr int KC = 128;            // contraction bytes staged per iteration (one cache line per trace row)
constexpr int STAGE_BYTES = TILE * KC;                 // one operand tile in LDS
constexpr int SYRK_LDS_BYTES = 2 * 2 * STAGE_BYTES;    // double buffer x (A, B) = 128 KiB

// 16-byte chunk c of row r lives at chunk position c ^ ((r >> 1) & 7).  The LDS has 64 four-byte banks,
// so a 16-byte access is served 16 lanes at a time; the 16 rows such a group touches when it reads one
// logical chunk then fall into 16 different 16-byte bank groups (row parity picks the half, the
// swizzled chunk the slot), and a 128-byte row written by 8 lanes stays one contiguous line.
__device__ __forceinline__ int lds_off(int row, int chunk) { return row * KC + ((chunk ^ ((row >> 1) & 7)) << 4); }

// C tile of 256 x 256 per workgroup; 4 waves in a 2 x 2 arrangement, each owning 128 x 128 =
// 4 x 4 MFMA tiles (256 accumulator registers).  The contraction runs in 128-byte chunks (four
// 32-byte MFMA k-steps) through a two-deep LDS ring fed from registers: chunk c+2 is in flight from
// memory into registers, chunk c+1 is being written into the idle LDS buffer, chunk c feeds the
// matrix cores; operand fragments of k-step s+1 are read from LDS while the 16 MFMAs of k-step s
// run.  (Direct-to-LDS loads were measured slower here: their LDS writes arrive 64 bytes per clock
// and, together with the fragment reads, saturate the LDS port.)
// Workgroups are numbered so that the eight L2 slices (one per XCD, workgroups are dealt to them
// round-robin) each walk a contiguous run of the tile schedule.
template <int MODE, bool VEC>
__global__ __launch_bounds__(256, 1) void coact_syrk_kernel(const int8_t* __restrict__ At, int N, int Npad, int64_t Tpad,
                                                            int32_t* __restrict__ C, uint32_t decay_q16, int nt,
                                                            int tiles_per_head, int total_tiles, int per_xcd,
                                                            const int32_t* __restrict__ tile_order) {
    extern __shared__ __attribute__((aligned(16))) int8_t lds[];
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int t = xcd * per_xcd + slot;
    if (slot >= per_xcd || t >= total_tiles) return;
    const int h = t / tiles_per_head;
    const int32_t packed = tile_order[t - h * tiles_per_head];
    const int ti = packed >> 16, tj = packed & 0xffff;
    const bool diag = ti == tj;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wy = wave >> 1, wx = wave & 1;

    // memory -> registers -> LDS: thread t moves 16-byte chunk t%8 of rows t/8 + 32*i, i = 0..7, of both
    // operand tiles (8 lanes cover one 128-byte line of a trace row).  The registers hold chunk c+2
    // while chunk c+1 sits in the idle LDS buffer and chunk c feeds the matrix cores.
    const int srow = tid >> 3, schunk = tid & 7;
    const int8_t* a_src = At + ((size_t)h * Npad + (size_t)ti * TILE + srow) * Tpad + schunk * 16;
    const int8_t* b_src = At + ((size_t)h * Npad + (size_t)tj * TILE + srow) * Tpad + schunk * 16;
    const size_t row32 = (size_t)32 * Tpad;
    const int nchunks = (int)(Tpad / KC);
    const int st_base = lds_off(srow, schunk);              // rows srow + 32*i share the swizzle term: constant byte offsets
    v4i sta[2][8], stb[2][8];                               // two register sets, indexed by chunk parity
    // loads number l0 .. l1-1 of the 16 that make up one chunk (0..7: A rows, 8..15: B rows)
    auto load_part = [&](int set, int chunk, int l0, int l1) {
        const int64_t k0 = (int64_t)min(chunk, nchunks - 1) * KC;      // clamped: a redundant reload past the end is harmless
#pragma unroll
        for (int l = l0; l < l1; ++l) {
            if (l < 8) sta[set][l] = *reinterpret_cast<const v4i*>(a_src + l * row32 + k0);
            else stb[set][l - 8] = *reinterpret_cast<const v4i*>(b_src + (l - 8) * row32 + k0);
        }
    };
    auto store_a = [&](int set, int buf) {
        int8_t* la = lds + buf * 2 * STAGE_BYTES + st_base;
#pragma unroll
        for (int i = 0; i < 8; ++i) *reinterpret_cast<v4i*>(la + i * 32 * KC) = sta[set][i];
    };
    auto store_b = [&](int set, int buf) {
        int8_t* lb = lds + buf * 2 * STAGE_BYTES + STAGE_BYTES + st_base;
#pragma unroll
        for (int i = 0; i < 8; ++i) *reinterpret_cast<v4i*>(lb + i * 32 * KC) = stb[set][i];
    };

    v16i acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // fragment addressing: lane l reads row l%32 of an MFMA tile, bytes [16*(l/32), +16) of the 32-byte
    // k-step.  The swizzle term only depends on the k-step; the tile index is a constant byte offset.
    const int frow = lane & 31, fhalf = lane >> 5;
    int fa_base[4], fb_base[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        fa_base[ks] = lds_off(wy * 128 + frow, 2 * ks + fhalf);
        fb_base[ks] = STAGE_BYTES + lds_off(wx * 128 + frow, 2 * ks + fhalf);
    }
    v4i fa[2][4], fb[2][4];
    auto read_frags = [&](int buf, int ks, int set) {
        const int8_t* base = lds + buf * 2 * STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            fa[set][i] = *reinterpret_cast<const v4i*>(base + fa_base[ks] + i * 32 * KC);
            fb[set][i] = *reinterpret_cast<const v4i*>(base + fb_base[ks] + i * 32 * KC);
        }
    };
    auto mfma16 = [&](int set) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[set][i], fb[set][j], acc[i][j], 0, 0, 0);
    };
    auto mfma_half = [&](int set, int half_idx) {
#pragma unroll
        for (int i = 2 * half_idx; i < 2 * half_idx + 2; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[set][i], fb[set][j], acc[i][j], 0, 0, 0);
    };
    // Scheduling hint for one k-step of 16 MFMAs: after MFMA i comes one fragment read (i < 8), one LDS
    // store (i >= 8, when the step carries stores) and one global load after every fourth MFMA, so
    // that no unit sees a burst.
    auto interleave16 = [&](bool with_stores) {
        _Pragma("unroll") for (int i = 0; i < 16; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (i < 8) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            else if (with_stores) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
            if ((i & 3) == 3) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
    };

    load_part(0, 0, 0, 16);
    load_part(1, 1, 0, 16);
    store_a(0, 0);
    store_b(0, 0);
    load_part(0, 2, 0, 4);
    __syncthreads();
    read_frags(0, 0, 0);

    // Chunk c computes out of LDS buffer c%2.  Register set (c+1)%2 holds chunk c+1: it is written to the
    // other LDS buffer during the second and third k-step and starts refilling with chunk c+3 in the
    // fourth.  Register set c%2 keeps refilling with chunk c+2 during the first three k-steps.  The 16
    // loads of a chunk are thus spread one per four MFMAs over a whole chunk time, and land at least a
    // chunk time before they are needed.  The hand-over barrier sits 8 MFMAs before the end of the
    // chunk; those last 8 MFMAs cover the LDS latency of the next chunk's first fragments.
    auto chunk_body = [&](int c, int buf) {                 // buf = c % 2, passed as a literal
        const int nset = buf ^ 1;
        read_frags(buf, 1, 1);
        load_part(buf, c + 2, 4, 8);
        mfma16(0);
        interleave16(false);

        read_frags(buf, 2, 0);
        store_a(nset, nset);                   // the other buffer was last read before the previous barrier
        load_part(buf, c + 2, 8, 12);
        mfma16(1);
        interleave16(true);

        read_frags(buf, 3, 1);
        store_b(nset, nset);
        load_part(buf, c + 2, 12, 16);
        mfma16(0);
        interleave16(true);

        load_part(nset, c + 3, 0, 4);
        mfma_half(1, 0);
        _Pragma("unroll") for (int g = 0; g < 4; ++g) {
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        read_frags(nset, 0, 0);                // after the last chunk this reads stale but valid LDS and is never used
        __builtin_amdgcn_sched_barrier(0);
        mfma_half(1, 1);
    };
    for (int c = 0; c < nchunks; c += 2) {                  // nchunks is even
        chunk_body(c, 0);
        chunk_body(c + 1, 1);
    }

    // 32x32 result layout: lane l, register r -> column l%32, row 8*(r/4) + 4*(l/32) + r%4.  One
    // register of a wave is therefore two whole 128-byte lines of the direct tile (32 consecutive
    // columns of two rows): the direct tile leaves straight from the accumulators in 4-byte stores,
    // with nothing to wait for.  In the mirrored tile a lane's register quadruple is 16 contiguous
    // bytes but the lines are spread over lanes, so that tile is re-laid out through the (now idle)
    // LDS and leaves in 16-byte stores that cover whole lines.  Streaming stores when C is not read.
    int32_t* Ch = C + (size_t)h * N * N;
    const int col_in = lane & 31, half = lane >> 5, row_in = half * 4;
    auto rmw1 = [&](int32_t* p, int32_t v) {
        if (MODE == 0) __builtin_nontemporal_store(v, p);
        else if (MODE == 1) *p += v;
        else *p = decayed(*p, decay_q16) + v;
    };
    auto rmw4 = [&](int32_t* p, v4i v) {
        if (MODE == 0) {
            __builtin_nontemporal_store(v, reinterpret_cast<v4i*>(p));
        } else {
            const v4i o = *reinterpret_cast<const v4i*>(p);
            if (MODE == 1) v += o;
            else {
                v.x += decayed(o.x, decay_q16); v.y += decayed(o.y, decay_q16);
                v.z += decayed(o.z, decay_q16); v.w += decayed(o.w, decay_q16);
            }
            *reinterpret_cast<v4i*>(p) = v;
        }
    };
    constexpr int TROW = 512 + 16;                                       // padded: 16-byte accesses of 16 lanes hit 16 bank groups
    int8_t* tbuf = lds + wave * (32 * TROW);
    const int gi_base = ti * TILE + wy * 128;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int gj_base = tj * TILE + wx * 128 + j * 32;
        // park the 128 x 32 block as [column][row] for the mirrored tile; the LDS executes one wave's
        // accesses in order, so the block of the previous j has been read by then
        if (VEC && !diag) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int rq = 0; rq < 4; ++rq) {
                    const v4i v = {acc[i][j][rq * 4], acc[i][j][rq * 4 + 1], acc[i][j][rq * 4 + 2], acc[i][j][rq * 4 + 3]};
                    *reinterpret_cast<v4i*>(tbuf + col_in * TROW + (i * 32 + rq * 8 + row_in) * 4) = v;
                }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        }
        // direct tile: rows gi_base + 0..127, columns gj_base + 0..31
        const int gjc = gj_base + col_in;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int gi = gi_base + i * 32 + (r >> 2) * 8 + row_in + (r & 3);
                if (gi < N && gjc < N) {
                    rmw1(Ch + (size_t)gi * N + gjc, acc[i][j][r]);
                    if (!VEC && !diag) rmw1(Ch + (size_t)gjc * N + gi, acc[i][j][r]);    // rows of C not 16-byte aligned: element-wise mirror
                }
            }
            if (MODE != 0) asm volatile("" ::: "memory");
        }
        // mirrored tile: rows gj_base + 0..31, columns gi_base + 0..127
        if (VEC && !diag) {
#pragma unroll
            for (int sidx = 0; sidx < 16; ++sidx) {
                const int r = 2 * sidx + half;
                const v4i v = *reinterpret_cast<const v4i*>(tbuf + r * TROW + col_in * 16);
                const int gj = gj_base + r, gi = gi_base + col_in * 4;
                if (gj < N && gi < N) rmw4(Ch + (size_t)gj * N + gi, v);
                if ((sidx & 7) == 7) asm volatile("" ::: "memory");
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
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

// Order in which the upper-triangle tiles are handed out: super-blocks of 4 x 8 tiles, so that the
// ~32 workgroups resident on one XCD share 4 A panels and 8 B panels in its L2.
static swarm_status ensure_tile_order(swarm_ctx* ctx, int nt) {
    if (ctx->tile_order && ctx->tile_order_nt == nt) return SWARM_OK;
    const size_t count = (size_t)nt * (nt + 1) / 2;
    int32_t* host = static_cast<int32_t*>(malloc(count * sizeof(int32_t)));
    if (!host) return SWARM_ENOMEM;
    size_t n = 0;
    for (int bi = 0; bi < nt; bi += 4)
        for (int bj = bi / 8 * 8; bj < nt; bj += 8)
            for (int ti = bi; ti < bi + 4 && ti < nt; ++ti)
                for (int tj = (bj > ti ? bj : ti); tj < bj + 8 && tj < nt; ++tj) host[n++] = (ti << 16) | tj;
    swarm_status st = SWARM_OK;
    if (n != count) {
        snprintf(ctx->err, sizeof(ctx->err), "coact: tile order covers %zu of %zu tiles", n, count);
        st = SWARM_EINVAL;
    }
    if (st == SWARM_OK) {
        size_t have = ctx->tile_order ? (size_t)ctx->tile_order_nt * (ctx->tile_order_nt + 1) / 2 * 4 : 0;
        st = swarm_grow(ctx, reinterpret_cast<void**>(&ctx->tile_order), &have, count * 4);
    }
    if (st == SWARM_OK) {
        hipError_t e = hipMemcpyAsync(ctx->tile_order, host, count * 4, hipMemcpyHostToDevice, ctx->stream);
        if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
        if (e != hipSuccess) {
            snprintf(ctx->err, sizeof(ctx->err), "coact: tile order upload failed: %s", hipGetErrorString(e));
            st = SWARM_EHIP;
        } else {
            ctx->tile_order_nt = nt;
        }
    }
    free(host);
    return st;
}

swarm_status launch_coact_syrk(swarm_ctx* ctx, int H, int N, int Npad, int64_t Tpad, int32_t* C, uint32_t decay_q16) {
    const int nt = Npad / TILE;
    const int64_t tiles_per_head = (int64_t)nt * (nt + 1) / 2;
    const int64_t total = tiles_per_head * H;
    if (total > (int64_t)1 << 30 || nt > 32767) {
        snprintf(ctx->err, sizeof(ctx->err), "coact: N=%d, H=%d give too many tiles for one launch", N, H);
        return SWARM_EINVAL;
    }
    swarm_status st = ensure_tile_order(ctx, nt);
    if (st != SWARM_OK) return st;
    const int per_xcd = (int)((total + 7) / 8);
    const int mode = decay_q16 == 0u ? 0 : decay_q16 == 65536u ? 1 : 2;
    const bool vec = (N & 3) == 0;
    using kernel_t = void (*)(const int8_t*, int, int, int64_t, int32_t*, uint32_t, int, int, int, int, const int32_t*);
    static const kernel_t kernels[3][2] = {{coact_syrk_kernel<0, false>, coact_syrk_kernel<0, true>},
                                           {coact_syrk_kernel<1, false>, coact_syrk_kernel<1, true>},
                                           {coact_syrk_kernel<2, false>, coact_syrk_kernel<2, true>}};
    static bool lds_opt_in = false;
    if (!lds_opt_in) {
        for (int m = 0; m < 3; ++m)
            for (int v = 0; v < 2; ++v) {
                const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernels[m][v]),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, SYRK_LDS_BYTES);
                if (e != hipSuccess) {
                    snprintf(ctx->err, sizeof(ctx->err), "coact: cannot opt in to %d bytes of LDS: %s", SYRK_LDS_BYTES, hipGetErrorString(e));
                    return SWARM_EHIP;
                }
            }
        lds_opt_in = true;
    }
    dim3 grid((unsigned)(per_xcd * 8)), block(256);
    const int tph = (int)tiles_per_head, tot = (int)total;
    hipLaunchKernelGGL(kernels[mode][vec ? 1 : 0], grid, block, SYRK_LDS_BYTES, ctx->stream,
                       static_cast<const int8_t*>(ctx->trace), N, Npad, Tpad, C, decay_q16, nt, tph, tot, per_xcd,
                       static_cast<const int32_t*>(ctx->tile_order));
    return swarm_check_launch(ctx, "coact_syrk_kernel");
}
