// Activation trace and co-activation accumulation (Section 5.1, Step 1): C[i][j] = number of trace
// rows in which entries i and j are both activated, i.e. C = A^T A for the binary trace A.
//
// The trace is binary, so it is kept in memory as bits: for every head and every run of 128 trace
// rows one 16-byte word per entry, bits[h][run][entry], one bit per trace row of the run (rows 32w ..
// 32w+31 in dword w, in the order of trace_bit below).  Both operands of the product are entry panels of this one array.  On the way
// to the matrix cores the bits are expanded to 4-bit 0/1 operands -- the 256 tile rows by the workgroup, into LDS
// (contraction index contiguous), the 64 tile columns of a wave by the wave itself, in registers -- and the product
// runs on the 4-bit form of v_mfma_f32_32x32x64_f8f6f4, exact for these operands (see below).  Feeding expanded
// operands from memory instead would multiply the traffic through the L2 by four to eight; the bit form keeps a
// smaller tile affordable.
// C is symmetric, so only tiles on or above the diagonal are computed and each off-diagonal tile is
// stored twice (once transposed).
#include <stdlib.h>

#include <type_traits>

#include "common.h"

namespace {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

// Position, inside its 32-bit word, of the bit of trace row r (0..31) of the word's group: row 8q + b is
// bit 4b + q, i.e. eight consecutive rows are the same bit of the word's eight nibbles.  Any fixed order
// serves the counts (both operands of a product, and both sides of an AND + popcount, use the same one);
// this one makes the expansion to 4-bit operands a shift and a mask.
__device__ __forceinline__ int trace_bit(int r) { return 4 * (r & 7) + (r >> 3); }

constexpr int TRACE_SPAN = 8192;   // entries one trace-building workgroup covers (128 KiB of LDS)

// One workgroup per (run of 128 trace rows, head, span of entries): the 128 selections are merged
// into an LDS image of the run's bit words, which then leaves as one contiguous, fully written block
// (no separate clearing pass, no global atomics).
// COUNT: also count, per trace row, the bits this workgroup sets for the first time (= the row's number
// of distinct valid entries inside the span) and add them to row_count[h][run * 128 + row].
template <bool COUNT>
__global__ __launch_bounds__(1024) void trace_build_kernel(const int32_t* __restrict__ idx, int64_t rows, int H, int k, int N,
                                                           int Npad, int nruns, uint4* __restrict__ bits,
                                                           uint32_t* __restrict__ dev_flags, int32_t* __restrict__ row_count) {
    extern __shared__ __attribute__((aligned(16))) uint32_t words[];          // [span][4], then 128 row counters when COUNT
    const int run = blockIdx.x, h = blockIdx.y;
    const int e0 = blockIdx.z * TRACE_SPAN;
    const int span = min(TRACE_SPAN, Npad - e0);
    uint32_t* fresh = words + span * 4;
    for (int i = threadIdx.x; i < span; i += blockDim.x) reinterpret_cast<uint4*>(words)[i] = make_uint4(0u, 0u, 0u, 0u);
    if (COUNT && threadIdx.x < 128) fresh[threadIdx.x] = 0u;
    __syncthreads();
    const int64_t row0 = (int64_t)run * 128;
    const int nrows = (int)min((int64_t)128, rows - row0);                       // <= 0 for a run of pure padding
    bool bad = false;
    // the run's nrows x k selected ids as one flat list: every thread busy, four independent loads in flight
    const int total = nrows > 0 ? nrows * k : 0;
    const int64_t row_stride = (int64_t)H * k;
    const int32_t* sel0 = idx + (row0 * H + h) * (int64_t)k;
    for (int i0 = threadIdx.x; i0 < total; i0 += 4 * blockDim.x) {
        int32_t e[4];
        int s[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = i0 + u * blockDim.x;
            s[u] = i / k;
            e[u] = i < total ? sel0[s[u] * row_stride + (i - s[u] * k)] : -1;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (i0 + u * (int)blockDim.x >= total) continue;
            if (e[u] < 0 || e[u] >= N) bad = true;
            else if (e[u] >= e0 && e[u] < e0 + span) {
                const uint32_t bit = 1u << trace_bit(s[u] & 31);
                if (COUNT) {
                    const bool first = !(atomicOr(&words[(e[u] - e0) * 4 + (s[u] >> 5)], bit) & bit);
                    // the lanes of a wave mostly work on one trace row (k consecutive list items): one add per wave then
                    const int s0 = __builtin_amdgcn_readfirstlane(s[u]);
                    if (__builtin_amdgcn_ballot_w64(s[u] != s0) == 0) {
                        const uint64_t firsts = __builtin_amdgcn_ballot_w64(first);
                        if (firsts && (threadIdx.x & 63) == (unsigned)__builtin_ctzll(__builtin_amdgcn_ballot_w64(true)))
                            atomicAdd(&fresh[s0], (uint32_t)__builtin_popcountll(firsts));
                    } else if (first) {
                        atomicAdd(&fresh[s[u]], 1u);
                    }
                } else {
                    atomicOr(&words[(e[u] - e0) * 4 + (s[u] >> 5)], bit);
                }
            }
        }
    }
    if (bad && blockIdx.z == 0) atomicOr(dev_flags, SWARM_DEV_BAD_ENTRY);
    __syncthreads();
    uint4* out = bits + ((size_t)h * nruns + run) * Npad + e0;
    const uint4* src = reinterpret_cast<const uint4*>(words);
    for (int i = threadIdx.x; i < span; i += blockDim.x) out[i] = src[i];
    if (COUNT && threadIdx.x < 128 && fresh[threadIdx.x])
        atomicAdd(&row_count[((size_t)h * nruns + run) * 128 + threadIdx.x], (int32_t)fresh[threadIdx.x]);
}

__global__ void fill_i32_kernel(int32_t* __restrict__ p, size_t n, int32_t v) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
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

// Updated count for the accumulating (MODE 1) and decayed (MODE 2) forms: v >= 0 is added to the old
// count or to its decayed value.  A sum that passes INT32_MAX wraps and sets `ovf`.
template <int MODE>
__device__ __forceinline__ int32_t updated_count(int32_t old, int32_t v, uint32_t decay_q16, bool& ovf) {
    const int32_t base = MODE == 1 ? old : decayed(old, decay_q16);
    const int32_t s = (int32_t)((uint32_t)base + (uint32_t)v);
    ovf |= s < base;
    return s;
}

constexpr int TM = 128;                        // C tile rows per workgroup
constexpr int TN = 128;                        // C tile columns per workgroup
constexpr int KC = 64;                         // contraction BYTES per chunk and operand row: 128 trace rows as 4-bit values, two MFMA k-steps of 64
constexpr int A_BYTES = TM * KC;               // A operand panel of one chunk in LDS: 8 KiB; two of them form the ring
constexpr int RAW_DEPTH = 4;                   // chunks of raw trace bits on their way from memory or waiting in LDS
constexpr int RAW_CHUNK = (TM + TN) * 16;      // one chunk of raw bits: the 16-byte run words of the tile's 128 rows, then of its 128 columns
constexpr int RAW_BASE = 2 * A_BYTES;          // the raw ring sits behind the operand ring
constexpr int SYRK_WAVES = 4;                  // 2 x 2 waves of 64 x 64
constexpr int TROW = 256 + 16;                 // epilogue staging row (64 counts), padded: the 16-byte slots of 8 consecutive lanes differ
constexpr int SYRK_LDS_BYTES = SYRK_WAVES * 32 * TROW;   // 34 KiB: the epilogue's staging (one 32-column block per wave) is the larger user
static_assert(SYRK_LDS_BYTES >= RAW_BASE + RAW_DEPTH * RAW_CHUNK, "operand ring and raw ring must fit");

// Operand rows in LDS are 64 bytes; 16-byte piece c of row r lives at slot c ^ swz(r).  Measured on
// gfx950: a 16-byte LDS read is served 16 consecutive lanes at a time across 64 four-byte banks, a
// 16-byte write 8 consecutive lanes at a time with only address bits 4..6 telling lanes apart.
// Fragment reads take one piece of 16 consecutive rows, so rows that agree in bits 0..1 need
// different swz; the expansion writes of 8 consecutive lanes cover 8 rows (A panel: thread = row)
// or 4 rows x 2 halves (B panel), so rows that agree in bit 0 within 8 need different swz, and bit 0
// of swz must follow bit 1 of the row.  swz = (bit1 ^ bit3) | bit2 << 1 does all of it.
__device__ __forceinline__ int lds_swz(int row) { return (((row >> 1) ^ (row >> 3)) & 1) | (((row >> 2) & 1) << 1); }
__device__ __forceinline__ int lds_off(int row, int piece) { return row * KC + ((piece ^ lds_swz(row)) << 4); }

// The matrix-core instruction is v_mfma_f32_32x32x64_f8f6f4 in its 4-bit form (E2M1): 0 and 1 are
// exact in it, products of them are exact, and the fp32 accumulators hold every integer up to 2^24
// exactly -- a call accumulates at most 2^24 trace rows, so the counts are exact, at twice the rate of
// the int8 instruction and with half the operand bytes.  Lane l of an operand holds row l%32, contraction
// indices [32 (l/32), +32) as 32 nibbles (16 bytes); 0.5, 1.0 and 2.0 are the nibbles 0b0001, 0b0010, 0b0100.
// No block scales (the unscaled form of the instruction: measured 3 % faster in the contraction loop than the scaled
// form with both scales 2^0, same results).
// Expansion of trace bits to nibbles: the rows of a 32-row group sit in their word so that the eight
// consecutive rows of an output dword are the same bit of the word's eight nibbles (trace_bit above),
// and a mask (with a shift where the bit has to move inside its nibble) is the whole expansion of eight rows.

// C tile of 128 x 128 per workgroup of 4 waves (2 x 2, each 64 x 64 = 2 x 2 MFMA tiles, 64 accumulator registers),
// four workgroups per compute unit, i.e. four waves per SIMD, each from a workgroup of its own.  A workgroup alternates
// between contracting (matrix cores) and writing its tile (memory); with equal demand on both, two workgroups per
// compute unit keep the busier of the two resources occupied two thirds of the time, four of them four fifths, and
// while one writes, every SIMD still has three waves feeding its matrix cores.  (Measured on one device with a model
// of this loop: two computing waves per SIMD run it at 69 % of the matrix cores' rate, one wave alone at 50 %.)
// The contraction runs in chunks of 128 trace rows (one 16-byte run word per entry).  Three stages, all in LDS:
//   raw ring   (RAW_DEPTH chunks)  the run words of the tile's 128 rows and 128 columns, loaded memory -> LDS directly
//              (buffer_load ... lds, 16 bytes per lane: one load per chunk and wave, no register ever holds data in
//              flight -- with four waves per SIMD there are none to spare for that)
//   row ring   (2 chunks)          the 128 rows expanded to 4-bit operands, thread t expands half of row t/2
//   fragments                      rows from the row ring (16-byte LDS reads), columns expanded in registers from the
//                                  lane's own 8 raw bytes per 32-column block
// One barrier per chunk hands over all three: before it a wave has waited for its own load of chunk d + 2, has written
// its share of chunk d + 1's rows and has read everything it needs of chunk d + 1's raw bits; after it the slot of
// chunk d + 1's raw bits is free for the load of chunk d + 1 + RAW_DEPTH, chunk d + 1's rows may be read, and the row
// buffer of chunk d may be overwritten (during chunk d + 1).
// Because the operands travel as bits, the small tile costs next to nothing in memory traffic.
// Workgroups are numbered so that the eight L2 slices (one per XCD, workgroups are dealt to them
// round-robin) each walk a contiguous run of the tile schedule.
// RHO (MODE 0, VEC): the epilogue also counts, for every row of C, the elements that reach the head's
// threshold cstar[h] (Algorithm 1, Step 3: the density of an entry is the number of entries within the
// radius, and "within the radius" is "count >= threshold", see the density pass).  A lane's register
// column of the direct tile gives the counts of the mirrored tile's rows, the mirrored tile's vectors
// give those of the direct tile's rows; a diagonal tile is computed in full, and by
// symmetry its column counts are its row counts.  Counts meet in LDS and leave as one
// atomic add per row and tile.
typedef __attribute__((address_space(3))) void lds_void;

template <int MODE, bool VEC, bool RHO = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 4)))
void coact_syrk_kernel(const v4i* __restrict__ bits, int N, int Npad, int nruns, int32_t* __restrict__ C, uint32_t decay_q16,
                       int tiles_per_head, int total_tiles, int per_xcd, const int32_t* __restrict__ tile_order,
                       uint32_t* __restrict__ dev_flags, const int64_t* __restrict__ cstar, int32_t* __restrict__ rho) {
    static_assert(!RHO || (MODE == 0 && VEC), "the fused density count belongs to the overwriting, vectorised form");
    extern __shared__ __attribute__((aligned(16))) int8_t lds[];
    const int xcd = blockIdx.x & 7, slot_id = blockIdx.x >> 3;
    const int t = xcd * per_xcd + slot_id;
    if (slot_id >= per_xcd || t >= total_tiles) return;
    const int h = t / tiles_per_head;
    const int32_t packed = tile_order[t - h * tiles_per_head];
    const int ti = packed >> 16, tj = packed & 0xffff;       // tile row, tile column (tj >= ti)
    const bool diag = tj == ti;                              // a diagonal tile is computed in full: no mirror

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wy = wave >> 1, wx = wave & 1;
    const int frow = lane & 31, fhalf = lane >> 5;

    // memory -> raw ring.  A chunk's raw bits are 4 KiB, contiguous in memory in two pieces (rows, columns), and land in
    // LDS in the same order: waves 0 and 1 bring rows [64 w, +64) of the tile, waves 2 and 3 columns [64 (w - 2), +64); lane l
    // of a load carries 16 bytes to byte 16 l of the wave's KiB.  One buffer descriptor per run (its range is the run:
    // 16 Npad bytes), so an offset past the run would read zeros, not memory.
    const char* panel = reinterpret_cast<const char*>(bits) + (size_t)h * nruns * Npad * 16;
    const uint32_t src_lane = (uint32_t)(((wave < 2 ? ti * TM + wave * 64 : tj * TN + (wave - 2) * 64) + lane) * 16);
    const int last_run = nruns - 1;
    auto issue_load = [&](int run) __attribute__((always_inline)) {                   // clamped: a redundant reload past the end is harmless
        {
            const char* runp = panel + (size_t)min(run, last_run) * Npad * 16;
            const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(runp), 0, Npad * 16, 0x00020000);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void*)(lds + RAW_BASE + (run % RAW_DEPTH) * RAW_CHUNK + wave * 1024), 16,
                                                     src_lane, 0, 0, 0);
        }
    };
    // raw ring -> registers.  Thread t owns half ahalf = t % 2 of row t / 2 of the row panel: 8 bytes, two pieces of 32 trace
    // rows.  Lane l of a fragment supplies row l % 32 with the contraction indices of lane half l / 32, and which 32 trace
    // rows of a chunk those are is free as long as both operands agree: k-step ks of lane half f is word 2 f + ks of the
    // run, so the two k-steps of a lane are 8 contiguous raw bytes.
    const int arow = tid >> 1, ahalf = tid & 1;
    const int rawa_off = RAW_BASE + arow * 16 + ahalf * 8;
    const int rawb_off = RAW_BASE + TM * 16 + (wx * 64 + frow) * 16 + fhalf * 8;
    v2i ba;                                        // raw bits of this thread's half row, next chunk
    v2i bw[2][2];                                  // raw column bits [chunk parity][column block] = {k-step 0, k-step 1}
    auto read_raw_a = [&](int run) __attribute__((always_inline)) {
        ba = *reinterpret_cast<const v2i*>(lds + (run % RAW_DEPTH) * RAW_CHUNK + rawa_off);
    };
    auto read_raw_b = [&](int set, int run) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < 2; ++j) bw[set][j] = *reinterpret_cast<const v2i*>(lds + (run % RAW_DEPTH) * RAW_CHUNK + rawb_off + j * 512);
    };
    // registers -> row ring, in pieces of 16 contraction bytes (32 trace rows = one 32-bit word of the run).  A piece is
    // expanded one dword (8 trace rows) at a time and stored when complete.
    int st_off[2];
#pragma unroll
    for (int p = 0; p < 2; ++p) st_off[p] = lds_off(arow, 2 * ahalf + p);
    v4i ex;
    // Row operand: the bit of trace row 8q + n of a 32-row word is bit q of nibble n, and for q = 0, 1, 2 it is left where
    // it is -- the nibbles 0b0001, 0b0010, 0b0100 are 0.5, 1 and 2 in E2M1 -- while the column operand (below) carries the
    // inverse factor at the same contraction index, so every product of two set bits is still exactly 1.  Only q = 3 (the
    // sign bit of its nibble) has to move.  Five vector operations per 32 trace rows instead of seven.
    auto expand_quarter = [&](int piece, int q) __attribute__((always_inline)) {
        const uint32_t w = (uint32_t)ba[piece];
        ex[q] = (int)(q == 3 ? (w >> 2) & 0x22222222u : w & (0x11111111u << q));
    };
    auto store_piece = [&](int buf, int piece) __attribute__((always_inline)) {
        *reinterpret_cast<v4i*>(lds + buf * A_BYTES + st_off[piece]) = ex;
    };

    v16f facc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) facc[i][j][r] = 0.f;

    // A fragment addressing: lane l reads row l%32 of an MFMA tile, the 16-byte piece 2 (l/32) + ks of its row.
    // The swizzle term is the same for rows 32 apart; the tile index is a constant byte offset.
    int fa_base[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) fa_base[ks] = lds_off(wy * 64 + frow, 2 * fhalf + ks);
    v4i fa[2][2], fb[2];
    auto read_a = [&](int buf, int ks, int fs, int i) __attribute__((always_inline)) {
        fa[fs][i] = *reinterpret_cast<const v4i*>(lds + buf * A_BYTES + fa_base[ks] + i * 32 * KC);
    };
    // Column operand: 2, 1, 0.5 and 1 at q = 0, 1, 2, 3, the inverses of the row operand's factors (two shifts, four masks).
    // One set of fragment registers: a k-step's columns are expanded after the previous k-step's MFMAs have been issued.
    auto expand_b = [&](int set, int ks, int j) __attribute__((always_inline)) {
        const uint32_t w = (uint32_t)bw[set][j][ks], w2 = w >> 2;
        fb[j] = v4i{(int)((w << 2) & 0x44444444u), (int)(w & 0x22222222u), (int)(w2 & 0x11111111u), (int)(w2 & 0x22222222u)};
    };
    // no block scales: with both scales 0 the compiler emits the unscaled form of the instruction (scale 2^0)
    auto mfma = [&](int fs, int m) __attribute__((always_inline)) {
        const v4i a4 = fa[fs][m >> 1], b4 = fb[m & 1];
        const v8i a8 = {a4.x, a4.y, a4.z, a4.w, 0, 0, 0, 0}, b8 = {b4.x, b4.y, b4.z, b4.w, 0, 0, 0, 0};   // the 4-bit form reads 4 registers
        facc[m >> 1][m & 1] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, facc[m >> 1][m & 1], 4, 4, 0, 0, 0, 0);
    };

    // start-up: chunks 0 .. RAW_DEPTH-1 on their way; chunk 0 expanded; chunk RAW_DEPTH into the slot of chunk 0
#pragma unroll
    for (int c = 0; c < RAW_DEPTH; ++c) issue_load(c);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    read_raw_a(0);
    read_raw_b(0, 0);
#pragma unroll
    for (int piece = 0; piece < 2; ++piece) {
#pragma unroll
        for (int q = 0; q < 4; ++q) expand_quarter(piece, q);
        store_piece(0, piece);
    }
    __syncthreads();
    issue_load(RAW_DEPTH);
#pragma unroll
    for (int i = 0; i < 2; ++i) read_a(0, 0, 0, i);
#pragma unroll
    for (int j = 0; j < 2; ++j) expand_b(0, 0, j);

    // Chunk d (parity `set`, passed as a literal) computes out of row buffer `set`.  First k-step: its four MFMAs, between
    // them the row fragments of the second k-step and this thread's share of chunk d + 1's rows (raw bits read at the top of
    // the chunk: they were published by the previous barrier); then the columns of the second k-step; the barrier; the load
    // of chunk d + 1 + RAW_DEPTH; the first row fragments of chunk d + 1, whose LDS latency the second k-step's MFMAs and
    // the SIMD's other waves cover; the columns of chunk d + 1's first k-step.
    auto chunk_body = [&](int d, int set) __attribute__((always_inline)) {
        const int nset = set ^ 1;
        read_raw_a(d + 1);
        read_raw_b(nset, d + 1);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            mfma(0, s);
            if (s < 2) read_a(set, 1, 1, s);
#pragma unroll
            for (int u = 2 * s; u < 2 * (s + 1); ++u) {
                expand_quarter(u >> 2, u & 3);
                if ((u & 3) == 3) store_piece(nset, u >> 2);
            }
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) expand_b(set, 1, j);
        // this wave's load of chunk d + 2 has landed; the RAW_DEPTH - 2 younger ones may still be in flight
        asm volatile("s_waitcnt vmcnt(%0)" :: "n"(RAW_DEPTH - 2) : "memory");
        __syncthreads();
        issue_load(d + 1 + RAW_DEPTH);
#pragma unroll
        for (int i = 0; i < 2; ++i) read_a(nset, 0, 0, i);            // after the last chunk this reads stale but valid LDS and is never used
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int s = 0; s < 4; ++s) mfma(1, s);
#pragma unroll
        for (int j = 0; j < 2; ++j) expand_b(nset, 0, j);
    };
    __builtin_amdgcn_s_setprio(2);                          // the contraction outranks the other waves' epilogue stores
    for (int d = 0; d < nruns; d += 2) {                    // nruns is a multiple of 4
        chunk_body(d, 0);
        chunk_body(d + 1, 1);
    }
    // every load has landed before the staging below reuses the rings, and every wave has left the loop
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    __builtin_amdgcn_s_setprio(0);
    // 32x32 result layout: lane l, register r -> column l%32, row 8*(r/4) + 4*(l/32) + r%4.  One
    // register of a wave is therefore two whole 128-byte lines of the direct tile (32 consecutive
    // columns of two rows): the direct tile leaves straight from the accumulators in 4-byte stores,
    // with nothing to wait for.  In the mirrored tile a lane's register quadruple is 16 contiguous
    // bytes but the lines are spread over lanes, so that tile is re-laid out through the (now idle)
    // LDS and leaves in 16-byte stores that cover whole lines.  Streaming stores when C is not read.
    // the counts as integers (exact: every partial sum is an integer below 2^24)
    v16i acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = (int32_t)facc[i][j][r];
    int32_t* Ch = C + (size_t)h * N * N;
    const int col_in = lane & 31, half = lane >> 5, row_in = half * 4;
    int8_t* tbuf = lds + wave * (32 * TROW);
    const int gi_base = ti * TM + wy * 64;
    const int mrow = lane >> 4, c16 = lane & 15;             // mirrored tile: a store covers 4 rows of 64 columns, 16 bytes per lane
    // Addresses are a wave-uniform row pointer (scalar arithmetic) plus one per-lane element offset
    // that is the same for every store of a tile.
    // The lane part is a 32-bit BYTE offset, so that an access is "scalar base + 32-bit lane offset", the
    // addressing form that needs no per-store 64-bit vector arithmetic and no register pair per address.
    const uint32_t lane_direct = ((uint32_t)row_in * (uint32_t)N + col_in) * 4u;
    const uint32_t lane_mirror = ((uint32_t)mrow * (uint32_t)N + c16 * 4) * 4u;
    auto at = [](int32_t* base, uint32_t byte_off) __attribute__((always_inline)) {
        return reinterpret_cast<int32_t*>(reinterpret_cast<char*>(base) + byte_off);
    };
    // density counters behind everything else in LDS: 128 direct-tile rows, then 128 direct-tile columns
    uint32_t* cnt_row = reinterpret_cast<uint32_t*>(lds + SYRK_LDS_BYTES);
    uint32_t* cnt_col = cnt_row + TM;
    int32_t c32 = 0x7fffffff;                              // counts never reach it (rows <= 2^24): "nothing is within the radius"
    if (RHO) {
        const int64_t c = cstar[h];
        if (c < 0x7fffffffll) c32 = (int32_t)c;
        if (threadIdx.x < TM) cnt_row[threadIdx.x] = 0u;
        else if (threadIdx.x < TM + TN) cnt_col[threadIdx.x - TM] = 0u;
        __syncthreads();                                   // the waves' counts meet in these counters
    }
    // 1 where v >= c32, 0 elsewhere, without a compare: counts lie in [0, 2^24] and c32 in [0, 2^31), so
    // (c32 - 1) - v cannot wrap and is negative exactly when v >= c32 (plain arithmetic: the compare form
    // kept its lane masks in scalar registers until those ran out)
    const int32_t c32m1 = c32 - 1;
    auto reaches = [&](int32_t v) __attribute__((always_inline)) { return (uint32_t)(c32m1 - v) >> 31; };
    uint32_t rowc[4] = {0u, 0u, 0u, 0u};
    bool ovf = false;
    auto combine = [&](int32_t old, int32_t v) __attribute__((always_inline)) {
        return updated_count<MODE == 0 ? 1 : MODE>(old, v, decay_q16, ovf);
    };
    // GUARD: the tile reaches past N (only tiles of the last tile row / column when N is not a multiple of 128)
    auto emit = [&](auto guard_tag) __attribute__((always_inline)) {
        constexpr bool GUARD = decltype(guard_tag)::value;
        // Overwriting form: the direct tile first, the two 32-column blocks of a row back to back, so that the two
        // 128-byte halves of a 256-byte run reach the memory system together.
        constexpr bool PAIRED = MODE == 0 && VEC;
        if (PAIRED) {
            int32_t* Cd = Ch + (size_t)gi_base * N + tj * TN + wx * 64;               // wave-uniform
            const bool c0_ok = !GUARD || tj * TN + wx * 64 + col_in < N, c1_ok = !GUARD || tj * TN + wx * 64 + 32 + col_in < N;
            uint32_t colc0 = 0u, colc1 = 0u;
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int urow = i * 32 + (r >> 2) * 8 + (r & 3);
                    int32_t* p = Cd + (size_t)urow * N;
                    if (!GUARD || gi_base + urow + row_in < N) {
                        if (c0_ok) __builtin_nontemporal_store(acc[i][0][r], at(p, lane_direct));
                        if (c1_ok) __builtin_nontemporal_store(acc[i][1][r], at(p + 32, lane_direct));
                        if (RHO && c0_ok) colc0 += reaches(acc[i][0][r]);
                        if (RHO && c1_ok) colc1 += reaches(acc[i][1][r]);
                    }
                }
            if (RHO) {
                atomicAdd(&cnt_col[wx * 64 + col_in], colc0);
                atomicAdd(&cnt_col[wx * 64 + 32 + col_in], colc1);
            }
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int gj_base = tj * TN + wx * 64 + j * 32;
            // park the 64 x 32 block as [column][row] for the mirrored tile; the LDS executes one wave's
            // accesses in order, so the block of the previous j has been read by then
            if (VEC && !diag) {
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int rq = 0; rq < 4; ++rq) {
                        const v4i v = {acc[i][j][rq * 4], acc[i][j][rq * 4 + 1], acc[i][j][rq * 4 + 2], acc[i][j][rq * 4 + 3]};
                        *reinterpret_cast<v4i*>(tbuf + col_in * TROW + (i * 32 + rq * 8 + row_in) * 4) = v;
                    }
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            }
            // direct tile: rows gi_base + 0..63, columns gj_base + 0..31
            size_t cj_off = (size_t)gi_base * N + gj_base;                            // wave-uniform
            if (RHO) asm volatile("" : "+s"(cj_off));   // own row pointers per column block: shared ones (128 scalar registers) do not fit beside the counting
            int32_t* Cj = Ch + cj_off;
            const bool col_ok = !GUARD || gj_base + col_in < N;
            uint32_t colc = 0u;
#pragma unroll
            for (int ip = 0; ip < (PAIRED ? 0 : 2); ip += 2) {                        // 32 rows x 2 in flight when C is read back
                int32_t old[2][16];
                if (MODE != 0) {
#pragma unroll
                    for (int i = ip; i < ip + 2; ++i)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int urow = i * 32 + (r >> 2) * 8 + (r & 3);
                            if (col_ok && (!GUARD || gi_base + urow + row_in < N)) old[i - ip][r] = *at(Cj + (size_t)urow * N, lane_direct);
                        }
                }
#pragma unroll
                for (int i = ip; i < ip + 2; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int urow = i * 32 + (r >> 2) * 8 + (r & 3);
                        int32_t* p = Cj + (size_t)urow * N;
                        if (col_ok && (!GUARD || gi_base + urow + row_in < N)) {
                            if (MODE == 0) __builtin_nontemporal_store(acc[i][j][r], at(p, lane_direct));
                            else *at(p, lane_direct) = combine(old[i - ip][r], acc[i][j][r]);
                            if (RHO) colc += reaches(acc[i][j][r]);
                            if (!VEC && !diag) {                                      // rows of C not 16-byte aligned: element-wise mirror
                                int32_t* q = Ch + (size_t)(gj_base + col_in) * N + gi_base + urow + row_in;
                                if (MODE == 0) *q = acc[i][j][r];
                                else *q = combine(*q, acc[i][j][r]);
                            }
                        }
                    }
                if (MODE != 0) asm volatile("" ::: "memory");
            }
            if (RHO && !PAIRED) atomicAdd(&cnt_col[wx * 64 + j * 32 + col_in], colc);
            // mirrored tile: rows gj_base + 0..31, columns gi_base + 0..63
            if (VEC && !diag) {
                size_t cm_off = (size_t)gj_base * N + gi_base;                        // wave-uniform
                if (RHO) asm volatile("" : "+s"(cm_off));
                int32_t* Cm = Ch + cm_off;
                const bool mcol_ok = !GUARD || gi_base + c16 * 4 < N;                 // N is a multiple of 4 here
                constexpr int MB = MODE == 0 ? 8 : 4;                                 // rows in flight: the old counts need registers too
#pragma unroll
                for (int sp = 0; sp < 8; sp += MB) {
                    v4i v[MB], o[MB];
#pragma unroll
                    for (int sidx = sp; sidx < sp + MB; ++sidx) {
                        v[sidx - sp] = *reinterpret_cast<const v4i*>(tbuf + (4 * sidx + mrow) * TROW + c16 * 16);
                        if (MODE != 0 && mcol_ok && (!GUARD || gj_base + 4 * sidx + mrow < N))
                            o[sidx - sp] = *reinterpret_cast<const v4i*>(at(Cm + (size_t)(4 * sidx) * N, lane_mirror));
                    }
#pragma unroll
                    for (int sidx = sp; sidx < sp + MB; ++sidx) {
                        if (mcol_ok && (!GUARD || gj_base + 4 * sidx + mrow < N)) {
                            v4i* p = reinterpret_cast<v4i*>(at(Cm + (size_t)(4 * sidx) * N, lane_mirror));
                            if (RHO) {
                                const v4i w = v[sidx - sp];
                                rowc[0] += reaches(w.x); rowc[1] += reaches(w.y); rowc[2] += reaches(w.z); rowc[3] += reaches(w.w);
                            }
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
    if (MODE == 0 && (ti + 1) * TM <= N && (tj + 1) * TN <= N) emit(std::false_type{});   // whole tile inside C: no per-store checks
    else emit(std::true_type{});
    if (MODE != 0 && ovf) atomicOr(dev_flags, SWARM_DEV_OVERFLOW);
    if (RHO) {
        if (!diag) {
#pragma unroll
            for (int c = 0; c < 4; ++c) atomicAdd(&cnt_row[wy * 64 + c16 * 4 + c], rowc[c]);
        }
        __syncthreads();
        int32_t* rh = rho + (size_t)h * N;
        const int u = threadIdx.x;
        if (!diag && u < TM && ti * TM + u < N && cnt_row[u]) atomicAdd(rh + ti * TM + u, (int32_t)cnt_row[u]);
        if (u >= TM && u < TM + TN && tj * TN + u - TM < N && cnt_col[u - TM]) atomicAdd(rh + tj * TN + u - TM, (int32_t)cnt_col[u - TM]);
    }
}

// The same counts without the matrix cores: C[i][j] = sum over the trace's 32-bit words of
// popcount(bits_i & bits_j), on the plain vector ALUs (v_and + v_bcnt, which adds the popcount to
// its accumulator).  A cross-check of the matrix-core path by an independent route, and its
// competitor: an eighth of the LDS traffic per trace row, but 2 ALU operations per 32 products
// where the matrix cores do 65536 per instruction.
// Workgroup = 64 x 64 tile of C on or above the diagonal, thread = 4 x 4 outputs (rows ty + 16 i,
// columns tx + 16 j), eight runs of 128 trace rows staged in LDS per pass.
constexpr int PT = 64, PRUNS = 8;

template <int MODE>
__global__ __launch_bounds__(256) void coact_popcount_kernel(const v4i* __restrict__ bits, int N, int Npad, int nruns,
                                                             int32_t* __restrict__ C, uint32_t decay_q16,
                                                             uint32_t* __restrict__ dev_flags) {
    __shared__ v4i sa[PRUNS][PT], sb[PRUNS][PT];
    const int h = blockIdx.z, ti = blockIdx.y, tj = blockIdx.x;
    if (tj < ti) return;
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const v4i* panel = bits + (size_t)h * nruns * Npad;
    uint32_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0u;
    for (int r0 = 0; r0 < nruns; r0 += PRUNS) {
        __syncthreads();
        for (int u = tid; u < PRUNS * PT; u += 256) {
            const int r = r0 + u / PT, e = u % PT;
            const v4i zero = {0, 0, 0, 0};
            sa[u / PT][e] = r < nruns ? panel[(size_t)r * Npad + ti * PT + e] : zero;
            sb[u / PT][e] = r < nruns ? panel[(size_t)r * Npad + tj * PT + e] : zero;
        }
        __syncthreads();
#pragma unroll 2
        for (int r = 0; r < PRUNS; ++r) {
            v4i a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = sa[r][ty + 16 * i]; b[i] = sb[r][tx + 16 * i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] += __popc((uint32_t)(a[i].x & b[j].x)) + __popc((uint32_t)(a[i].y & b[j].y)) +
                                 __popc((uint32_t)(a[i].z & b[j].z)) + __popc((uint32_t)(a[i].w & b[j].w));
        }
    }
    int32_t* Ch = C + (size_t)h * N * N;
    bool ovf = false;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int gi = ti * PT + ty + 16 * i, gj = tj * PT + tx + 16 * j;
            if (gi >= N || gj >= N) continue;
            const int32_t v = (int32_t)acc[i][j];
            int32_t* p = Ch + (size_t)gi * N + gj;
            int32_t* q = Ch + (size_t)gj * N + gi;
            if (MODE == 0) { *p = v; if (ti != tj) *q = v; }
            else {
                *p = updated_count<MODE == 0 ? 1 : MODE>(*p, v, decay_q16, ovf);
                if (ti != tj) *q = updated_count<MODE == 0 ? 1 : MODE>(*q, v, decay_q16, ovf);
            }
        }
    if (MODE != 0 && ovf) atomicOr(dev_flags, SWARM_DEV_OVERFLOW);
}

}  // namespace

swarm_status launch_trace_build(swarm_ctx* ctx, const int32_t* idx, int64_t rows, int H, int k, int N, int Npad,
                                int nruns, uint32_t flags, int32_t* row_count) {
    if (flags & SWARM_CHECK_IDX) {
        hipLaunchKernelGGL(check_distinct_kernel, dim3((unsigned)(rows * H)), dim3(256), 0, ctx->stream, idx, k,
                           ctx->dev_flags);
        const swarm_status st = swarm_check_launch(ctx, "check_distinct_kernel");
        if (st != SWARM_OK) return st;
    }
    const int span = Npad < TRACE_SPAN ? Npad : TRACE_SPAN;
    const size_t lds_bytes = (size_t)span * 16 + (row_count ? 512 : 0);
    if (!ctx->trace_lds_opt_in) {                          // per context: the attribute belongs to the device the context is bound to
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&trace_build_kernel<false>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, TRACE_SPAN * 16);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&trace_build_kernel<true>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, TRACE_SPAN * 16 + 512);
        if (e != hipSuccess) {
            snprintf(ctx->err, sizeof(ctx->err), "coact: cannot opt in to %d bytes of LDS: %s", TRACE_SPAN * 16 + 512, hipGetErrorString(e));
            return SWARM_EHIP;
        }
        ctx->trace_lds_opt_in = true;
    }
    const dim3 grid((unsigned)nruns, (unsigned)H, (unsigned)((Npad + TRACE_SPAN - 1) / TRACE_SPAN));
    if (row_count) {
        const size_t n = (size_t)H * nruns * 128;
        hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)((n + 1023) / 1024 < 1024 ? (n + 1023) / 1024 : 1024)), dim3(1024), 0,
                           ctx->stream, row_count, n, 0);
        const swarm_status st = swarm_check_launch(ctx, "fill_i32_kernel");
        if (st != SWARM_OK) return st;
        hipLaunchKernelGGL(trace_build_kernel<true>, grid, dim3(1024), lds_bytes, ctx->stream, idx, rows, H, k, N, Npad, nruns,
                           reinterpret_cast<uint4*>(ctx->trace), ctx->dev_flags, row_count);
    } else {
        hipLaunchKernelGGL(trace_build_kernel<false>, grid, dim3(1024), lds_bytes, ctx->stream, idx, rows, H, k, N, Npad, nruns,
                           reinterpret_cast<uint4*>(ctx->trace), ctx->dev_flags, row_count);
    }
    return swarm_check_launch(ctx, "trace_build_kernel");
}

// Order in which the tiles on or above the diagonal are handed out: super-blocks of 8 x 16 tiles
// (1024 x 2048 entries), so that the workgroups resident on one XCD share few panels in its L2.
// Tile (ti, tj) covers rows [128 ti, +128) and columns [128 tj, +128), tj >= ti.
static swarm_status tile_order_for(swarm_ctx* ctx, int ntm, const int32_t** out) {
    for (const auto& t : ctx->tile_orders)
        if (t.first == ntm) { *out = t.second; return SWARM_OK; }
    if (ctx->capturing) {
        snprintf(ctx->err, sizeof(ctx->err), "coact: first call with this N while recording; run the sequence once first");
        return SWARM_EINVAL;
    }
    const size_t count = (size_t)ntm * (ntm + 1) / 2;
    int32_t* host = static_cast<int32_t*>(malloc(count * sizeof(int32_t)));
    if (!host) {
        snprintf(ctx->err, sizeof(ctx->err), "out of host memory");
        return SWARM_ENOMEM;
    }
    size_t n = 0;
    for (int bi = 0; bi < ntm; bi += 8)
        for (int bj = bi / 16 * 16; bj < ntm; bj += 16)
            for (int ti = bi; ti < bi + 8 && ti < ntm; ++ti)
                for (int tj = (bj > ti ? bj : ti); tj < bj + 16 && tj < ntm; ++tj)
                    if (n < count) host[n++] = (ti << 16) | tj; else ++n;
    swarm_status st = SWARM_OK;
    int32_t* dev = nullptr;
    if (n != count) {
        snprintf(ctx->err, sizeof(ctx->err), "coact: tile order covers %zu of %zu tiles", n, count);
        st = SWARM_EINVAL;
    }
    if (st == SWARM_OK) {
        hipError_t e = hipMalloc(reinterpret_cast<void**>(&dev), count * sizeof(int32_t));
        if (e == hipSuccess) e = hipMemcpyAsync(dev, host, count * sizeof(int32_t), hipMemcpyHostToDevice, ctx->stream);
        if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
        if (e == hipSuccess) {
            try {
                ctx->tile_orders.emplace_back(ntm, dev);
            } catch (...) {
                e = hipErrorOutOfMemory;
            }
        }
        if (e != hipSuccess) {
            (void)hipGetLastError();
            snprintf(ctx->err, sizeof(ctx->err), "coact: tile order set-up failed: %s", hipGetErrorString(e));
            if (dev) (void)hipFree(dev);
            st = SWARM_EHIP;
        }
    }
    free(host);
    *out = dev;
    return st;
}

swarm_status launch_fill_i32(swarm_ctx* ctx, int32_t* p, size_t n, int32_t v) {
    hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)((n + 1023) / 1024 < 1024 ? (n + 1023) / 1024 : 1024)), dim3(1024), 0,
                       ctx->stream, p, n, v);
    return swarm_check_launch(ctx, "fill_i32_kernel");
}

// cstar and rho both null: plain update of C.  Both given (overwriting form, N a multiple of 4 only): the
// epilogue adds to rho[h][i] the number of elements of row i that reach cstar[h]; rho must be zero.
swarm_status launch_coact_syrk(swarm_ctx* ctx, int H, int N, int Npad, int nruns, int32_t* C, uint32_t decay_q16,
                               const int64_t* cstar, int32_t* rho) {
    const int ntm = Npad / TM;
    const int64_t tiles_per_head = (int64_t)ntm * (ntm + 1) / 2;
    const int64_t total = tiles_per_head * H;
    if (total > (int64_t)1 << 30 || ntm > 65535) {
        snprintf(ctx->err, sizeof(ctx->err), "coact: N=%d, H=%d give too many tiles for one launch", N, H);
        return SWARM_EINVAL;
    }
    const int32_t* tile_order = nullptr;
    swarm_status st = tile_order_for(ctx, ntm, &tile_order);
    if (st != SWARM_OK) return st;
    const int per_xcd = (int)((total + 7) / 8);
    const int mode = decay_q16 == 0u ? 0 : decay_q16 == 65536u ? 1 : 2;
    const bool vec = (N & 3) == 0;
    const bool fused = cstar != nullptr;
    if (fused && (!rho || mode != 0 || !vec)) {
        snprintf(ctx->err, sizeof(ctx->err), "coact: the fused density count needs the overwriting form and N a multiple of 4");
        return SWARM_EINVAL;
    }
    using kernel_t = void (*)(const v4i*, int, int, int, int32_t*, uint32_t, int, int, int, const int32_t*, uint32_t*,
                              const int64_t*, int32_t*);
    static const kernel_t kernels[3][2] = {{coact_syrk_kernel<0, false>, coact_syrk_kernel<0, true>},
                                           {coact_syrk_kernel<1, false>, coact_syrk_kernel<1, true>},
                                           {coact_syrk_kernel<2, false>, coact_syrk_kernel<2, true>}};
    static const kernel_t fused_kernel = coact_syrk_kernel<0, true, true>;
    constexpr int RHO_LDS_BYTES = SYRK_LDS_BYTES + (TM + TN) * 4;
    if (!ctx->syrk_lds_opt_in) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fused_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                           RHO_LDS_BYTES);
        for (int m = 0; m < 3 && e == hipSuccess; ++m)
            for (int v = 0; v < 2 && e == hipSuccess; ++v)
                e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernels[m][v]), hipFuncAttributeMaxDynamicSharedMemorySize,
                                        SYRK_LDS_BYTES);
        if (e != hipSuccess) {
            snprintf(ctx->err, sizeof(ctx->err), "coact: cannot opt in to %d bytes of LDS: %s", RHO_LDS_BYTES, hipGetErrorString(e));
            return SWARM_EHIP;
        }
        ctx->syrk_lds_opt_in = true;
    }
    dim3 grid((unsigned)(per_xcd * 8)), block(64 * SYRK_WAVES);
    const int tph = (int)tiles_per_head, tot = (int)total;
    hipLaunchKernelGGL(fused ? fused_kernel : kernels[mode][vec ? 1 : 0], grid, block, fused ? RHO_LDS_BYTES : SYRK_LDS_BYTES,
                       ctx->stream, reinterpret_cast<const v4i*>(ctx->trace), N, Npad, nruns, C, decay_q16, tph, tot, per_xcd,
                       tile_order, ctx->dev_flags, cstar, rho);
    return swarm_check_launch(ctx, "coact_syrk_kernel");
}

swarm_status launch_coact_popcount(swarm_ctx* ctx, int H, int N, int Npad, int nruns, int32_t* C, uint32_t decay_q16) {
    const unsigned nt = (unsigned)(Npad / PT);
    if (nt > 65535u || H > 65535) {
        snprintf(ctx->err, sizeof(ctx->err), "coact: N=%d, H=%d too large for the popcount route", N, H);
        return SWARM_EINVAL;
    }
    const dim3 grid(nt, nt, (unsigned)H), block(256);
    const v4i* bits = reinterpret_cast<const v4i*>(ctx->trace);
    if (decay_q16 == 0u) hipLaunchKernelGGL(coact_popcount_kernel<0>, grid, block, 0, ctx->stream, bits, N, Npad, nruns, C, decay_q16, ctx->dev_flags);
    else if (decay_q16 == 65536u) hipLaunchKernelGGL(coact_popcount_kernel<1>, grid, block, 0, ctx->stream, bits, N, Npad, nruns, C, decay_q16, ctx->dev_flags);
    else hipLaunchKernelGGL(coact_popcount_kernel<2>, grid, block, 0, ctx->stream, bits, N, Npad, nruns, C, decay_q16, ctx->dev_flags);
    return swarm_check_launch(ctx, "coact_popcount_kernel");
}
