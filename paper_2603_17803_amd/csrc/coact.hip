// Activation trace and co-activation accumulation (Section 5.1, Step 1): C[i][j] = number of trace
// rows in which entries i and j are both activated, i.e. C = A^T A for the binary trace A.
//
// The trace is binary, so it is kept in memory as bits: for every head and every run of 128 trace
// rows ("chunk") one 16-byte word per entry, bits[h][chunk][entry], bit s = "entry activated in trace
// row 128*chunk + s".  Both operands of the product are entry panels of this one array.  On the way
// to the matrix cores a workgroup expands the bits of its two 256-entry panels to int8 0/1 rows in
// LDS (contraction index contiguous), and the product runs on v_mfma_i32_32x32x32_i8 with exact
// int32 accumulation.  Feeding int8 from memory instead would make every workgroup pull
// 512 bytes per contraction byte-step through the L2, which at this tile size is within 15% of
// the L2's bandwidth at full matrix-core rate; the bit form needs an eighth of it.
// C is symmetric, so only tiles on or above the diagonal are computed and each off-diagonal tile is
// stored twice (once transposed).
#include <stdlib.h>

#include <type_traits>

#include "common.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int TRACE_SPAN = 8192;   // entries one trace-building workgroup covers (128 KiB of LDS)

// One workgroup per (chunk, head, span of entries): the 128 selections of the chunk are merged into
// an LDS image of the chunk's bit words, which then leaves as one contiguous, fully written block
// (no separate clearing pass, no global atomics).
__global__ __launch_bounds__(1024) void trace_build_kernel(const int32_t* __restrict__ idx, int64_t rows, int H, int k, int N,
                                                           int Npad, int nchunks, uint4* __restrict__ bits,
                                                           uint32_t* __restrict__ dev_flags) {
    extern __shared__ __attribute__((aligned(16))) uint32_t words[];          // [span][4]
    const int chunk = blockIdx.x, h = blockIdx.y;
    const int e0 = blockIdx.z * TRACE_SPAN;
    const int span = min(TRACE_SPAN, Npad - e0);
    for (int i = threadIdx.x; i < span * 4; i += blockDim.x) words[i] = 0u;
    __syncthreads();
    const int64_t row0 = (int64_t)chunk * 128;
    const int nrows = (int)min((int64_t)128, rows - row0);                       // <= 0 for a chunk of pure padding
    bool bad = false;
    for (int s = 0; s < nrows; ++s) {
        const int32_t* sel = idx + ((row0 + s) * H + h) * (int64_t)k;
        for (int j = threadIdx.x; j < k; j += blockDim.x) {
            const int32_t e = sel[j];
            if (e < 0 || e >= N) bad = true;
            else if (e >= e0 && e < e0 + span) atomicOr(&words[(e - e0) * 4 + (s >> 5)], 1u << (s & 31));
        }
    }
    if (bad && blockIdx.z == 0) atomicOr(dev_flags, SWARM_DEV_BAD_ENTRY);
    __syncthreads();
    uint4* out = bits + ((size_t)h * nchunks + chunk) * Npad + e0;
    const uint4* src = reinterpret_cast<const uint4*>(words);
    for (int i = threadIdx.x; i < span; i += blockDim.x) out[i] = src[i];
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

// Operand rows in LDS are 128 bytes; 16-byte piece c of row r lives at slot c ^ swz(r).  Measured on
// gfx950: a 16-byte LDS read is served 16 consecutive lanes at a time across 64 four-byte banks, a
// 16-byte write 8 consecutive lanes at a time with only the slot (address bits 4..6) telling lanes
// apart.  Fragment reads take one piece of 16 consecutive rows, expansion writes one piece of 8
// consecutive rows (thread = row): swz must differ on rows of equal parity within 16 rows (reads:
// parity picks the bank half) and on all rows within 8 (writes).  swz(r) = bits 1..2 of r, with bit 2
// = bit 3 of r xor bit 0 of r, does both.
__device__ __forceinline__ int lds_swz(int row) { return ((row >> 1) & 3) | ((((row >> 3) ^ row) & 1) << 2); }
__device__ __forceinline__ int lds_off(int row, int chunk) { return row * KC + ((chunk ^ lds_swz(row)) << 4); }

// Expansion of trace bits to bytes of 0/1, four at a time: a nibble times (1 + 2^7 + 2^14 + 2^21) puts
// bit b at bit 8b (the four shifted copies do not overlap, so nothing carries); a mask drops the rest.

// C tile of 256 x 256 per workgroup; 4 waves in a 2 x 2 arrangement, each owning 128 x 128 =
// 4 x 4 MFMA tiles (256 accumulator registers).  The contraction runs in chunks of 128 trace rows
// (four 32-byte MFMA k-steps) through a two-deep LDS ring: thread t owns entry t of both panels; the
// 16-byte bit words of chunk c+2 and c+3 are in flight from memory, the words of chunk c+1 are
// being expanded and written into the idle LDS buffer, chunk c feeds the matrix cores; operand
// fragments of k-step s+1 are read from LDS while the 16 MFMAs of k-step s run.
// Workgroups are numbered so that the eight L2 slices (one per XCD, workgroups are dealt to them
// round-robin) each walk a contiguous run of the tile schedule.
template <int MODE, bool VEC>
__global__ __launch_bounds__(256, 1) void coact_syrk_kernel(const v4i* __restrict__ bits, int N, int Npad, int nchunks,
                                                            int32_t* __restrict__ C, uint32_t decay_q16,
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

    // memory -> registers: one 16-byte word per thread, panel and chunk.  Four register sets, indexed
    // by chunk number mod 4.
    const v4i* a_src = bits + (size_t)h * nchunks * Npad + (size_t)ti * TILE + tid;
    const v4i* b_src = bits + (size_t)h * nchunks * Npad + (size_t)tj * TILE + tid;
    v4i ba[4], bb[4];
    const size_t last_off = (size_t)(nchunks - 1) * Npad;
    auto load_a = [&](int set, int chunk) __attribute__((always_inline)) {            // clamped: a redundant reload past the end is harmless
        ba[set] = a_src[chunk < nchunks ? (size_t)chunk * Npad : last_off];
    };
    auto load_b = [&](int set, int chunk) __attribute__((always_inline)) {
        bb[set] = b_src[chunk < nchunks ? (size_t)chunk * Npad : last_off];
    };
    // registers -> LDS: piece p (0..7) of a panel row is 16 contraction bytes; pieces 8..15 are the B
    // panel's.  A piece is expanded one dword (4 trace rows) at a time and stored when complete.
    int st_off[8];
#pragma unroll
    for (int p = 0; p < 8; ++p) st_off[p] = lds_off(tid, p);
    v4i ex;
    auto expand_quarter = [&](int set, int piece, int q) __attribute__((always_inline)) {
        const int p = piece & 7;
        const uint32_t w = (uint32_t)(piece < 8 ? ba[set][p >> 1] : bb[set][p >> 1]);
        ex[q] = (int)(__umul24(__builtin_amdgcn_ubfe(w, 16 * (p & 1) + 4 * q, 4), 0x00204081u) & 0x01010101u);
    };
    auto store_piece = [&](int buf, int piece) __attribute__((always_inline)) {
        *reinterpret_cast<v4i*>(lds + buf * 2 * STAGE_BYTES + (piece < 8 ? 0 : STAGE_BYTES) + st_off[piece & 7]) = ex;
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
    // fragment number f of a k-step, in the order the MFMAs need them (MFMA m uses A tile m/4, B tile m%4)
    auto read_frag = [&](int buf, int ks, int set, int f) __attribute__((always_inline)) {
        const int8_t* base = lds + buf * 2 * STAGE_BYTES;
        if (f == 0) fa[set][0] = *reinterpret_cast<const v4i*>(base + fa_base[ks]);
        else if (f < 5) fb[set][f - 1] = *reinterpret_cast<const v4i*>(base + fb_base[ks] + (f - 1) * 32 * KC);
        else fa[set][f - 4] = *reinterpret_cast<const v4i*>(base + fa_base[ks] + (f - 4) * 32 * KC);
    };
    auto mfma = [&](int set, int m) __attribute__((always_inline)) {
        acc[m >> 2][m & 3] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[set][m >> 2], fb[set][m & 3], acc[m >> 2][m & 3], 0, 0, 0);
    };

    load_a(0, 0); load_b(0, 0);
    load_a(1, 1); load_b(1, 1);
    load_a(2, 2); load_b(2, 2);
#pragma unroll
    for (int piece = 0; piece < 16; ++piece) {
#pragma unroll
        for (int q = 0; q < 4; ++q) expand_quarter(0, piece, q);
        store_piece(0, piece);
    }
    __syncthreads();
#pragma unroll
    for (int f = 0; f < 8; ++f) read_frag(0, 0, 0, f);

    // Chunk c computes out of LDS buffer c%2; its own bit words (register set c%4) are spent.  Set
    // (c+1)%4 is expanded into the other LDS buffer, which no wave reads after the hand-over barrier
    // of chunk c-1; set (c+3)%4 is refilled at the start.  The work is laid out as 64 slots, one per
    // MFMA, fenced against reordering: slot m of a k-step issues the MFMA, then a fragment read for the
    // next k-step (m < 8), then its share of the expansion (64 dwords of 3 operations and 16 LDS
    // stores per chunk, spread over the first 56 slots) so that no unit sees a burst.  The hand-over
    // barrier sits 8 MFMAs before the end of the chunk; those last 8 MFMAs cover the LDS latency of
    // the next chunk's first fragments.
    auto chunk_body = [&](int c, int buf, int set) __attribute__((always_inline)) {   // buf = c % 2, set = c % 4, passed as literals
        const int nbuf = buf ^ 1, nset = (set + 1) & 3, lset = (set + 3) & 3;
#pragma unroll
        for (int slot = 0; slot < 56; ++slot) {
            const int ks = slot >> 4, m = slot & 15;
            mfma(ks & 1, m);
            if (ks < 3 && m < 8) read_frag(buf, ks + 1, (ks + 1) & 1, m);
            if (slot == 0) load_a(lset, c + 3);
            if (slot == 1) load_b(lset, c + 3);
            // quarters [slot*64/56, (slot+1)*64/56) of the 64
#pragma unroll
            for (int u = slot * 8 / 7; u < (slot + 1) * 8 / 7; ++u) {
                expand_quarter(nset, u >> 2, u & 3);
                if ((u & 3) == 3) store_piece(nbuf, u >> 2);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        __syncthreads();
#pragma unroll
        for (int f = 0; f < 8; ++f) read_frag(nbuf, 0, 0, f);          // after the last chunk this reads stale but valid LDS and is never used
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int m = 8; m < 16; ++m) mfma(1, m);
    };
    for (int c = 0; c < nchunks; c += 4) {                  // nchunks is a multiple of 4
        chunk_body(c, 0, 0);
        chunk_body(c + 1, 1, 1);
        chunk_body(c + 2, 0, 2);
        chunk_body(c + 3, 1, 3);
    }

    // 32x32 result layout: lane l, register r -> column l%32, row 8*(r/4) + 4*(l/32) + r%4.  One
    // register of a wave is therefore two whole 128-byte lines of the direct tile (32 consecutive
    // columns of two rows): the direct tile leaves straight from the accumulators in 4-byte stores,
    // with nothing to wait for.  In the mirrored tile a lane's register quadruple is 16 contiguous
    // bytes but the lines are spread over lanes, so that tile is re-laid out through the (now idle)
    // LDS and leaves in 16-byte stores that cover whole lines.  Streaming stores when C is not read.
    int32_t* Ch = C + (size_t)h * N * N;
    const int col_in = lane & 31, half = lane >> 5, row_in = half * 4;
    constexpr int TROW = 512 + 16;                                       // padded: the 16-byte slots of 8 consecutive lanes differ
    int8_t* tbuf = lds + wave * (32 * TROW);
    const int gi_base = ti * TILE + wy * 128;
    // Addresses are a wave-uniform row pointer (scalar arithmetic) plus one per-lane element offset
    // that is the same for every store of a tile.
    const uint32_t lane_direct = (uint32_t)row_in * (uint32_t)N + col_in;
    const uint32_t lane_mirror = (uint32_t)half * (uint32_t)N + col_in * 4;
    auto combine = [&](int32_t old, int32_t v) __attribute__((always_inline)) {
        return MODE == 1 ? old + v : decayed(old, decay_q16) + v;
    };
    // GUARD: the tile reaches past N (only tiles of the last tile row / column when N is not a multiple of 256)
    auto emit = [&](auto guard_tag) __attribute__((always_inline)) {
        constexpr bool GUARD = decltype(guard_tag)::value;
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
            int32_t* Cj = Ch + (size_t)gi_base * N + gj_base;                         // wave-uniform
            const bool col_ok = !GUARD || gj_base + col_in < N;
#pragma unroll
            for (int ip = 0; ip < 4; ip += 2) {                                       // 32 rows x 2 in flight when C is read back
                int32_t old[2][16];
                if (MODE != 0) {
#pragma unroll
                    for (int i = ip; i < ip + 2; ++i)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int urow = i * 32 + (r >> 2) * 8 + (r & 3);
                            if (col_ok && (!GUARD || gi_base + urow + row_in < N)) old[i - ip][r] = (Cj + (size_t)urow * N)[lane_direct];
                        }
                }
#pragma unroll
                for (int i = ip; i < ip + 2; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int urow = i * 32 + (r >> 2) * 8 + (r & 3);
                        int32_t* p = Cj + (size_t)urow * N;
                        if (col_ok && (!GUARD || gi_base + urow + row_in < N)) {
                            if (MODE == 0) __builtin_nontemporal_store(acc[i][j][r], p + lane_direct);
                            else p[lane_direct] = combine(old[i - ip][r], acc[i][j][r]);
                            if (!VEC && !diag) {                                      // rows of C not 16-byte aligned: element-wise mirror
                                int32_t* q = Ch + (size_t)(gj_base + col_in) * N + gi_base + urow + row_in;
                                if (MODE == 0) *q = acc[i][j][r];
                                else *q = combine(*q, acc[i][j][r]);
                            }
                        }
                    }
                if (MODE != 0) asm volatile("" ::: "memory");
            }
            // mirrored tile: rows gj_base + 0..31, columns gi_base + 0..127
            if (VEC && !diag) {
                int32_t* Cm = Ch + (size_t)gj_base * N + gi_base;                     // wave-uniform
                const bool mcol_ok = !GUARD || gi_base + col_in * 4 < N;              // N is a multiple of 4 here
#pragma unroll
                for (int sp = 0; sp < 16; sp += 8) {
                    v4i v[8], o[8];
#pragma unroll
                    for (int sidx = sp; sidx < sp + 8; ++sidx) {
                        v[sidx - sp] = *reinterpret_cast<const v4i*>(tbuf + (2 * sidx + half) * TROW + col_in * 16);
                        if (MODE != 0 && mcol_ok && (!GUARD || gj_base + 2 * sidx + half < N))
                            o[sidx - sp] = *reinterpret_cast<const v4i*>(Cm + (size_t)(2 * sidx) * N + lane_mirror);
                    }
#pragma unroll
                    for (int sidx = sp; sidx < sp + 8; ++sidx) {
                        if (mcol_ok && (!GUARD || gj_base + 2 * sidx + half < N)) {
                            v4i* p = reinterpret_cast<v4i*>(Cm + (size_t)(2 * sidx) * N + lane_mirror);
                            if (MODE == 0) __builtin_nontemporal_store(v[sidx - sp], p);
                            else {
                                v4i w = v[sidx - sp];
                                const v4i q = o[sidx - sp];
                                w.x = combine(q.x, w.x); w.y = combine(q.y, w.y); w.z = combine(q.z, w.z); w.w = combine(q.w, w.w);
                                *p = w;
                            }
                        }
                    }
                    if (MODE != 0) asm volatile("" ::: "memory");
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            }
        }
    };
    if (MODE == 0 && (ti + 1) * TILE <= N && (tj + 1) * TILE <= N) emit(std::false_type{});   // whole tile inside C: no per-store checks
    else emit(std::true_type{});
}

}  // namespace

swarm_status launch_trace_build(swarm_ctx* ctx, const int32_t* idx, int64_t rows, int H, int k, int N, int Npad,
                                int nchunks, uint32_t flags) {
    if (flags & SWARM_CHECK_IDX) {
        hipLaunchKernelGGL(check_distinct_kernel, dim3((unsigned)(rows * H)), dim3(256), 0, ctx->stream, idx, k,
                           ctx->dev_flags);
        const swarm_status st = swarm_check_launch(ctx, "check_distinct_kernel");
        if (st != SWARM_OK) return st;
    }
    const int span = Npad < TRACE_SPAN ? Npad : TRACE_SPAN;
    const size_t lds_bytes = (size_t)span * 16;
    static bool lds_opt_in = false;
    if (!lds_opt_in) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&trace_build_kernel),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, TRACE_SPAN * 16);
        if (e != hipSuccess) {
            snprintf(ctx->err, sizeof(ctx->err), "coact: cannot opt in to %d bytes of LDS: %s", TRACE_SPAN * 16, hipGetErrorString(e));
            return SWARM_EHIP;
        }
        lds_opt_in = true;
    }
    const dim3 grid((unsigned)nchunks, (unsigned)H, (unsigned)((Npad + TRACE_SPAN - 1) / TRACE_SPAN));
    hipLaunchKernelGGL(trace_build_kernel, grid, dim3(1024), lds_bytes, ctx->stream, idx, rows, H, k, N, Npad, nchunks,
                       reinterpret_cast<uint4*>(ctx->trace), ctx->dev_flags);
    return swarm_check_launch(ctx, "trace_build_kernel");
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

swarm_status launch_coact_syrk(swarm_ctx* ctx, int H, int N, int Npad, int nchunks, int32_t* C, uint32_t decay_q16) {
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
    using kernel_t = void (*)(const v4i*, int, int, int, int32_t*, uint32_t, int, int, int, const int32_t*);
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
                       reinterpret_cast<const v4i*>(ctx->trace), N, Npad, nchunks, C, decay_q16, tph, tot, per_xcd,
                       static_cast<const int32_t*>(ctx->tile_order));
    return swarm_check_launch(ctx, "coact_syrk_kernel");
}
