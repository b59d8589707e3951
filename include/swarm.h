/*
 * swarm.h -- C boundary of the MI355X hot path of co-activation-aware KV-cache offloading.
 *
 * The path, per decode step:
 *     score every KV entry (token key or page summary) against the query   (Section 2.3)
 *  -> keep the k highest-scoring entries                                   (Section 2.3)
 *  -> record the selection as one row of a binary activation trace
 *  -> count how often two entries are activated together, C = A^T A       (Section 5.1, Step 1)
 *  -> turn the step's selection into per-SSD request queues               (Section 6.1)
 * and, around that path: the density pass over C that starts the clustering (Section 5.1, Steps 1-3),
 * cluster maintenance over the local window (Section 6.2), and retrieval through the medoid index
 * (Section 5.2 Tier 1, Section 6.1).
 *
 * Conventions that hold for every call below:
 *  - Every data pointer is a DEVICE pointer owned by the caller.  The library never frees,
 *    reallocates or keeps a caller pointer after the call's work has run.
 *  - Work is enqueued on the context's HIP stream, in call order, and returns without waiting
 *    for it; results are valid once the caller has synchronised that stream.
 *  - Scratch memory belongs to the context and grows on demand.  Growing allocates (and
 *    synchronises the stream); a call whose shapes are no larger than those of an earlier call
 *    allocates nothing, so a warmed-up call sequence may be captured into a HIP graph.
 *  - The return value is the only host-side error channel.  Nothing throws or aborts.  Bad
 *    arguments give SWARM_EINVAL before anything is enqueued.  Bad *data* (an index outside
 *    its range) never makes a kernel read or write out of bounds: the offending item is
 *    skipped and a sticky flag is raised that swarm_device_status() reports.
 *  - A context belongs to the device it was created on; that device must be the calling thread's
 *    current device for every call (SWARM_EINVAL otherwise).  swarm_create makes it current.
 *  - One context per stream; a context is not thread-safe.  bf16 is the upper half of an IEEE
 *    binary32.  All integer arrays are int32 unless stated.
 */
#ifndef SWARM_H_
#define SWARM_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct swarm_ctx swarm_ctx;

typedef enum {
    SWARM_OK = 0,
    SWARM_EINVAL = -1,    /* argument rejected on the host; nothing was enqueued            */
    SWARM_ENOMEM = -2,    /* scratch allocation failed                                      */
    SWARM_EHIP = -3,      /* a HIP runtime call failed; text in swarm_last_error()          */
    SWARM_EOVERFLOW = -4, /* reserved (count overflow is detected on the device: SWARM_DEV_OVERFLOW) */
    SWARM_EDATA = -5      /* swarm_device_status(): a kernel met an out-of-range index      */
} swarm_status;

typedef enum {
    SWARM_KEYS_TOKEN = 0,       /* data: bf16 [H][N][d], one key per entry                   */
    SWARM_KEYS_PAGE_MINMAX = 1  /* data: bf16 [H][N][2][d], channel-wise min then max of the
                                   page's keys, 4*d contiguous bytes per page                */
} swarm_key_kind;

/* Key-side operand of the scoring step. */
typedef struct {
    int32_t kind;        /* swarm_key_kind                                                    */
    const void* data;    /* device, 16-byte aligned                                           */
    int32_t H;           /* KV heads                                                          */
    int32_t N;           /* scored entries (tokens or pages) per head                         */
    int32_t d;           /* head dimension: a multiple of 8, at most 512                      */
    int32_t G;           /* query heads per KV head (grouped-query attention), >= 1           */
} swarm_keys;

/* flags of swarm_coact_accumulate */
#define SWARM_CHECK_IDX 1u   /* validate range and distinctness of every selection on the device */
#define SWARM_COACT_POPCOUNT 2u /* count with AND + popcount on the vector ALUs instead of the matrix cores:
                                  same result by an independent route (cross-check, slower) */

/* bits of swarm_device_status()'s *flags */
#define SWARM_DEV_BAD_ENTRY   1u  /* entry id outside [0,N)                      */
#define SWARM_DEV_BAD_CLUSTER 2u  /* cluster id outside [0,Nc)                   */
#define SWARM_DEV_BAD_SSD     4u  /* replica slot >= D, or a cluster with none   */
#define SWARM_DEV_CAP         8u  /* a group had more distinct clusters than cap */
#define SWARM_DEV_DUP_ENTRY   16u /* repeated entry within one selection         */
#define SWARM_DEV_BAD_OFFSETS 32u /* bucket offsets not non-decreasing from 0 to at most cap */
#define SWARM_DEV_OVERFLOW    64u /* a co-activation count passed INT32_MAX (it wrapped) */

/* Creates a context bound to HIP device `device` and to `hip_stream` (a hipStream_t; NULL is the
 * default stream).  The stream stays the caller's.  */
swarm_status swarm_create(swarm_ctx** out, int device, void* hip_stream);
/* Frees the context and its scratch.  Synchronises the stream first. */
swarm_status swarm_destroy(swarm_ctx* ctx);
/* Text of the last error on this context (or of the last failed swarm_create when ctx is NULL).
 * Valid until the next call on the context.  */
const char* swarm_last_error(const swarm_ctx* ctx);
/* Hash of the sources this library was built from (set by the build script; "unknown" otherwise), so that
 * a binary left behind by an older tree can be told from a current one.  Static storage. */
const char* swarm_source_hash(void);
/* Synchronises the stream, reads and clears the sticky device flags.  Returns SWARM_OK when no
 * flag was set, SWARM_EDATA otherwise; *flags (nullable, host) receives the SWARM_DEV_* bits. */
swarm_status swarm_device_status(swarm_ctx* ctx, uint32_t* flags);

/*
 * Score + select (Section 2.3: every KV entry gets a relevance score against the query -- inner
 * products being the example the section names -- and the entries with the highest scores are kept).
 *
 *   token keys:      s[b][h][n] = sum_g sum_c q[b][h*G+g][c] * K[h][n][c]
 *   page summaries:  s[b][h][n] = sum_g sum_c max(q_c * min[h][n][c], q_c * max[h][n][c])
 *                    (channel-wise upper bound of the inner product over the page's box)
 *   Products of two bf16 values are exact in fp32 and are accumulated in fp32.  A page term is computed as
 *   min(q_c,0) * min_c + max(q_c,0) * max_c, which equals max(q_c * min_c, q_c * max_c) when the summary is finite
 *   and min_c <= max_c -- the precondition of page scoring: an infinite or NaN summary channel, or min_c > max_c,
 *   gives a score that differs from the formula above (a zero weight times an infinity is NaN).  With up to seven
 *   streams the G query heads of a group are first added into fp32 weights (one rounding per head), then multiplied;
 *   with eight or more streams every query head is its own exact bf16 operand of the bf16 matrix cores and the heads
 *   add in their fp32 accumulators.  Either way a score differs from the exact sum by fp32 accumulation error only.
 *   select: the k largest of s[b][h][0..N); equal scores are won by the lower index; -0 equals
 *   +0; NaN ranks below every number.  The k indices come out in ascending order.
 *
 * q           device, bf16 [B][H*G][d], 16-byte aligned.
 * B           decode streams scored in this call (>= 1); each gets its own selection.
 * k           1 <= k <= N.
 * out_idx     device, int32 [B][H][k].
 * out_scores  device, fp32 [B][H][N], or NULL to keep the scores in the context's scratch.
 * Errors: SWARM_EINVAL for a NULL required pointer, misaligned data/q, k outside [1,N], d not a
 * multiple of 8 or above 512, H/N/G/B < 1, N > 2^30, H > 65535, B*H > 2^24.
 */
swarm_status swarm_score_select(swarm_ctx* ctx, const swarm_keys* keys, const void* q, int32_t B, int32_t k,
                                int32_t* out_idx, float* out_scores);

/*
 * swarm_score_select for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same kernels and same results as swarm_score_select with
 * out_scores = NULL, but the scratch (fp32 scores [B][H][N] and the winners of the sliced selection of long
 * rows) lives in one static device array of
 * SWARM_STATIC_SCRATCH_BYTES per GPU, which the library holds from load until the process ends.  The call
 * allocates and frees nothing, on the device or through any library.
 * Every call on a GPU shares that GPU's array, on whatever context or stream: calls that overlap in time on
 * one GPU race (calls on one stream are ordered and safe).  The array keeps the last call's contents; nothing
 * needs clearing, every byte a kernel reads is written earlier in the same call.
 * Errors: those of swarm_score_select; SWARM_EINVAL when the shapes need more than the static scratch
 * (4*B*H*N bytes of scores, rounded up to 256, plus the slices' winners where used).
 */
#define SWARM_STATIC_SCRATCH_BYTES ((size_t)8 << 20)
swarm_status swarm_score_select_static(swarm_ctx* ctx, const swarm_keys* keys, const void* q, int32_t B, int32_t k,
                                       int32_t* out_idx);

/*
 * The scoring half of swarm_score_select on its own (Section 2.3, relevance scores): same formulas,
 * same arguments, no selection.  out_scores: device, fp32 [B][H][N], required.
 */
swarm_status swarm_score(swarm_ctx* ctx, const swarm_keys* keys, const void* q, int32_t B, float* out_scores);

/*
 * Co-activation accumulation (Section 5.1, Step 1: element (i,j) counts the number of times entries
 * i and j are activated together; the diagonal is an entry's own activation count).
 *
 * The `rows` selections are scattered into a binary trace A (rows x N per head, kept entry-major
 * as bits in the context's scratch, expanded to 4-bit 0/1 operands on the way to the matrix cores) and
 * C[h] is updated with A^T A computed exactly: the products of 0/1 operands are exact in the 4-bit form
 * of the matrix-core instruction, its fp32 accumulators hold integers exactly up to 2^24 (the most trace
 * rows a call accepts), and the update of C itself is int32 arithmetic:
 *     decay_q16 == 65536 : C += A^T A
 *     decay_q16 == 0     : C  = A^T A            (C is not read)
 *     otherwise          : C  = floor((C * decay_q16 + 2^15) / 2^16) + A^T A   (int64 intermediate)
 * The decayed form lets stale statistics fade when the workload drifts (the degradation of
 * co-activation statistics is the paper's fourth challenge, Section 3.2); the mechanism itself is
 * not in the paper.
 *
 * idx    device, int32 [rows][H][k]; within one (row, head) the k entries must be distinct and in
 *        [0,N) (any order).  Out-of-range entries are skipped and flagged.
 * rows   trace rows in this call (steps x streams since the last call), 1 <= rows <= 2^24.
 * H, N   1 <= H <= 65535, 1 <= N <= 2^20.
 * C      device, int32 [H][N][N] row-major, in/out, 16-byte aligned.
 * flags  SWARM_CHECK_IDX additionally flags repeated entries (SWARM_DEV_DUP_ENTRY); a repeated
 *        entry counts once either way, because the trace is binary.  SWARM_COACT_POPCOUNT computes the
 *        same counts as popcount(bits_i & bits_j) over the bit trace, without the matrix cores.
 * Counts are exact as long as they fit int32: rows <= 2^24 cannot overflow a fresh C, and when an
 * accumulating or decayed update passes INT32_MAX the count wraps and SWARM_DEV_OVERFLOW is raised.
 * Errors: SWARM_EINVAL as above or decay_q16 > 65536; SWARM_ENOMEM if the trace (H*N*rows/8 bytes,
 * rows rounded up to 512, N to 256) cannot be allocated.
 */
swarm_status swarm_coact_accumulate(swarm_ctx* ctx, const int32_t* idx, int64_t rows, int32_t H, int32_t k,
                                    int32_t N, int32_t* C, uint32_t decay_q16, uint32_t flags);

/*
 * Co-activation density and medoid queue (Section 5.1: the co-activation probability of Step 1, the
 * distance of Step 2, the density and the descending medoid queue of Algorithm 1's Step 3) -- the
 * streaming front half of the clustering, whose sequential expansion step stays on the host.
 *
 *   total[h] = sum over all (k, l) of C[h][k][l]     (or totals_in[h] when given, e.g. to rescale)
 *   P(i,j)   = C[h][i][j] / total[h] ;  d(i,j) = 1 - P(i,j)          (fp64, each operation rounded once)
 *   rho[h][i] = number of j with d(i,j) <= tau                       (Algorithm 1: every j, "<=")
 *   queue[h]  = entry ids in descending rho, equal rho in ascending id
 * SWARM_RHO_EXCLUDE_SELF leaves j = i out and SWARM_RHO_STRICT tests d < tau (the form of the paper's
 * density equation).  total = 0 leaves P undefined: no pair is counted.  Counts must be >= 0.
 *
 * C          device, int32 [H][N][N], 16-byte aligned (as produced by swarm_coact_accumulate).
 * totals_in  device, int64 [H], or NULL to sum C (one more pass over C).
 * rho        device out, int32 [H][N].
 * queue      device out, int32 [H][N], or NULL to skip the queue.
 * totals_out device out, int64 [H], or NULL.
 * Errors: SWARM_EINVAL for NULL C or rho, H/N < 1, misaligned pointers, unknown flags.
 */
#define SWARM_RHO_EXCLUDE_SELF 1u
#define SWARM_RHO_STRICT 2u
swarm_status swarm_coact_density(swarm_ctx* ctx, const int32_t* C, int32_t H, int32_t N, const int64_t* totals_in,
                                 double tau, uint32_t flags, int32_t* rho, int32_t* queue, int64_t* totals_out);

/*
 * Co-activation build and density pass in one go (Section 5.1, Steps 1-3): C = A^T A as
 * swarm_coact_accumulate computes it with decay_q16 = 0, and rho / queue / totals exactly as
 * swarm_coact_density would then compute them from that C with totals_in = NULL.  The grand total of
 * a fresh build is known before C exists (it is the sum over trace rows of the squared number of
 * activated entries), so the radius test "d(i,j) <= tau" is an integer threshold on the count and is
 * applied to every tile of C while it is still in registers: C is written once and never read back.
 * (When N is not a multiple of 4 the two steps run one after the other, with the same results.)
 *
 * idx, rows, H, k, N, C   as in swarm_coact_accumulate; C is overwritten.
 * flags                   SWARM_CHECK_IDX or 0.
 * tau, rho_flags, rho, queue, totals_out   as in swarm_coact_density (queue and totals_out may be NULL).
 * Errors: those of the two calls.
 */
swarm_status swarm_coact_build_density(swarm_ctx* ctx, const int32_t* idx, int64_t rows, int32_t H, int32_t k, int32_t N,
                                       int32_t* C, uint32_t flags, double tau, uint32_t rho_flags, int32_t* rho, int32_t* queue,
                                       int64_t* totals_out);

/*
 * Cluster maintenance over the local window (Section 6.2: the distance between a newly generated entry
 * and a cluster is 1 - f(e_new, m_i) / W, with f the number of the window's W steps in which the entry
 * and the cluster's medoid m_i are activated together; the entry joins every cluster whose distance is
 * below the radius, and is placed on that cluster's next SSD).
 *
 *   f[h][a][c]      = number of t < W with new_ids[h][a] and medoids[h][c] both in sel[t][h][0..k)
 *   member[h][a][c] = 1 - f / W < tau            (fp64; strict: the text asks for a distance below the radius)
 *   disk[h][a][c]   = (primary[h][c] + size[h][c] + j + 1) mod D for the j-th entry (in the order of
 *                     new_ids, j from 0) that joins cluster c, -1 where the entry does not join
 *                     (the cluster grows by one with every joining entry: a reading, the paper places
 *                     one entry at a time)
 * sel      device, int32 [W][H][k], the window's selections (1 <= W <= 2048).
 * new_ids  device, int32 [H][n_new];  medoids device, int32 [H][Nc]: entry ids in [0,N); an id outside
 *          the range counts as never activated and is flagged (SWARM_DEV_BAD_ENTRY).
 * primary, size  device, int32 [H][Nc] (first SSD and current entry count of each cluster), or both
 *          NULL when disk is NULL.
 * f_out    device out, int32 [H][n_new][Nc], or NULL.   member  device out, uint8 [H][n_new][Nc].
 * disk     device out, int32 [H][n_new][Nc], or NULL.
 * The window's trace is rebuilt in the context's scratch (it replaces the trace of the last
 * swarm_coact_accumulate).  Errors: SWARM_EINVAL for NULL required pointers or sizes out of range.
 */
swarm_status swarm_window_assign(swarm_ctx* ctx, const int32_t* sel, int32_t W, int32_t H, int32_t k, int32_t N,
                                 const int32_t* new_ids, int32_t n_new, const int32_t* medoids, int32_t Nc, double tau,
                                 const int32_t* primary, const int32_t* size, int32_t D, int32_t* f_out, uint8_t* member,
                                 int32_t* disk);

/*
 * Request mapping (Section 6.1: merge the activated clusters, drop what is already resident in
 * DRAM, then fill one bucket per SSD -- items in ascending order of replication factor, an item
 * with a single copy to its SSD, an item with several copies to the SSD whose bucket is currently
 * the smallest).  The routed unit is a cluster, the paper's atomic retrieval unit.
 *
 * For each group g (KV head = g % H):
 *   1. clusters = { e2c[head][e] : e in sel[g][0..S) } minus clusters whose bit is set in `resident`;
 *   2. visit them in ascending (replication factor, cluster id), the replication factor being the
 *      number of slots >= 0 in replicas[head*Nc + c][0..R);
 *   3. send each to the candidate SSD with the smallest load, ties to the smallest SSD id;
 *      load += weight[head*Nc + c] (1 when weight is NULL);
 *   4. emit the buckets SSD-major, each in insertion order.
 *
 * sel        device, int32 [groups][S] entry ids (repeats allowed; all streams of a step merged; -1 is
 *            padding and is skipped).
 * e2c        device, int32 [H][N] cluster of each entry, in [0,Nc).
 * replicas   device, int32 [H*Nc][R]: distinct SSD ids in [0,D); a slot < 0 is unused.
 * weight     device, int32 [H*Nc] or NULL.
 * resident   device, uint32 bitmap over head*Nc + c (bit i of word i/32), or NULL.
 * q_off      device out, int32 [groups][D+1]: bucket d of group g is q_cluster[g][q_off[g][d] .. q_off[g][d+1]).
 * q_cluster  device out, int32 [groups][cap]; slots past q_off[g][D] are set to -1.
 * q_load     device out, int32 [groups][D] final bucket loads.
 * cap        row length of q_cluster; min(S, Nc) always suffices.  A group with more distinct
 *            clusters than cap is truncated and flagged (SWARM_DEV_CAP).
 * weight entries must be >= 0 (negative ones count as 0).
 * Errors: SWARM_EINVAL for NULL required pointers, R < 1, R > D, D > 64, Nc > 2^20, cap < 1,
 * S/H/N/Nc/groups < 1, or on-chip staging too large: 24 * cap + Nc / 8 + 256 bytes must fit in 64 KiB.
 */
swarm_status swarm_map_requests(swarm_ctx* ctx, const int32_t* sel, int64_t groups, int32_t S, int32_t H, int32_t N,
                                const int32_t* e2c, int32_t Nc, const int32_t* replicas, int32_t R, int32_t D,
                                const int32_t* weight, const uint32_t* resident,
                                int32_t* q_off, int32_t* q_cluster, int32_t* q_load, int32_t cap);

/*
 * Request mapping of a batch of decode streams, straight from the selections (Section 6.1: the clusters activated
 * at a step are merged before the buckets are filled; Fig. 9's caption shows two queries' clusters merged).
 * Group (step, head) merges the entries idx[step][b][head][0..k) of all B streams b and is mapped exactly as
 * swarm_map_requests maps a group holding those B*k entries: same queues, bit for bit.
 *
 * idx     device, int32 [steps][B][H][k]: the out_idx of `steps` consecutive swarm_score_select calls of B streams.
 * outputs q_off [steps*H][D+1], q_cluster [steps*H][cap], q_load [steps*H][D]; everything else as in
 *         swarm_map_requests (S there is B*k here; cap = min(B*k, Nc) always suffices).
 * Errors: those of swarm_map_requests; SWARM_EINVAL for steps/B/k < 1, B*k > 2^24, H*k > 2^30, steps*H > 2^30.
 */
swarm_status swarm_map_requests_streams(swarm_ctx* ctx, const int32_t* idx, int64_t steps, int32_t B, int32_t H, int32_t k, int32_t N,
                                        const int32_t* e2c, int32_t Nc, const int32_t* replicas, int32_t R, int32_t D,
                                        const int32_t* weight, const uint32_t* resident,
                                        int32_t* q_off, int32_t* q_cluster, int32_t* q_load, int32_t cap);

/*
 * Medoid-indexed retrieval (Section 5.2, Tier 1: the medoid of each cluster is its index entry and is
 * scored against the query to decide whether the cluster is retrieved; Section 6.1: the activated
 * clusters are merged into the set of entries to transfer, which the mapping step routes entry by
 * entry; the finished buckets are submitted head by head).  Three calls around swarm_map_requests:
 *
 * swarm_score_select_indexed: as swarm_score_select, over the listed entries only.
 *   row_ids    device, int32 [H][M], entry ids in [0,N) (an id outside scores 0 and is flagged).
 *   scores     s[b][h][m] = score of entry row_ids[h][m]; out_scores fp32 [B][H][M] or NULL.
 *   out_idx    device, int32 [B][H][k]: positions m in the list (ascending), 1 <= k <= M.
 *
 * swarm_expand_clusters: per group g (head g % H) the distinct clusters of clusters[g][0..Sc) (-1 is
 *   padding) in ascending id, each replaced by its members cl_entries[h][cl_off[h][c] .. cl_off[h][c+1]):
 *   entries[g][0..count[g]), then -1 padding up to cap_e (too small a cap_e truncates and raises
 *   SWARM_DEV_CAP).  An entry held by several activated clusters appears once per cluster; merging into
 *   a set, and dropping DRAM-resident entries, is what swarm_map_requests then does (with Nc = N and the
 *   identity entry->cluster table it routes entries, replication factor = number of SSD copies).
 *   cl_off device int32 [H][Nc+1]; cl_entries device int32 [H][E]; Nc <= 2^18.
 *
 * swarm_submission_order: order[g] lists the items of swarm_map_requests' buckets batch by batch (batch
 *   b = the b-th item of every bucket that has one, ascending SSD id), -1 padded to cap;
 *   batch_off[g][b] is where batch b starts (entries from nb[g] on repeat the item count), int32
 *   [groups][cap+1]; nb[g] = number of batches = longest bucket.  q_off[g] must run from 0 in
 *   non-decreasing steps to at most cap; a group where it does not gets an empty order, nb = 0 and
 *   SWARM_DEV_BAD_OFFSETS.
 * In swarm_map_requests an entry id of -1 is padding and is skipped, so ragged entry lists can be mapped.
 */
swarm_status swarm_score_select_indexed(swarm_ctx* ctx, const swarm_keys* keys, const int32_t* row_ids, int32_t M, const void* q,
                                        int32_t B, int32_t k, int32_t* out_idx, float* out_scores);
swarm_status swarm_expand_clusters(swarm_ctx* ctx, const int32_t* clusters, int64_t groups, int32_t Sc, int32_t H, int32_t Nc,
                                   const int32_t* cl_off, const int32_t* cl_entries, int32_t E, int32_t* entries, int32_t* count,
                                   int32_t cap_e);
swarm_status swarm_submission_order(swarm_ctx* ctx, const int32_t* q_off, const int32_t* q_cluster, int64_t groups, int32_t D,
                                    int32_t cap, int32_t* order, int32_t* batch_off, int32_t* nb);

/*
 * One decode step of a single stream: swarm_score_select with B = 1 followed by swarm_map_requests on
 * that selection (groups = H, one per KV head; S = k), with identical results (Sections 2.3 and 6.1:
 * the entries activated at a step are what the step requests from the SSDs).  The step's three
 * stages depend on each other, so their cost is latency, not throughput; here selection and mapping
 * run in one kernel where the shapes allow it (the mapping's lookup tables load while the selection
 * runs), and otherwise as the two calls would.
 * Arguments as in swarm_score_select (q: bf16 [H*G][d]; out_idx: int32 [H][k]; out_scores fp32 [H][N]
 * or NULL) and swarm_map_requests (N = keys->N; q_off [H][D+1], q_cluster [H][cap], q_load [H][D]).
 * Errors: those of the two calls.
 */
swarm_status swarm_step(swarm_ctx* ctx, const swarm_keys* keys, const void* q, int32_t k, int32_t* out_idx,
                        float* out_scores, const int32_t* e2c, int32_t Nc, const int32_t* replicas, int32_t R, int32_t D,
                        const int32_t* weight, const uint32_t* resident, int32_t* q_off, int32_t* q_cluster,
                        int32_t* q_load, int32_t cap);

/*
 * Replay of a recorded call sequence.  The per-step work of the path is a handful of short kernels,
 * so a long step-sequential run is bounded by launch cost unless it is recorded once and replayed.
 * Between swarm_capture_begin and swarm_capture_end every entry point above records its kernels
 * into a HIP graph instead of running them (the context's stream must not be the NULL stream, and
 * the recorded calls must not need to grow scratch: run the same sequence once beforehand).
 * swarm_graph_launch enqueues one replay on the context's stream; pointers and shapes are those
 * of the recorded calls, so the caller keeps those buffers alive and refreshes their contents.
 * swarm_device_status must not be called while recording.  A recorded graph also refers to the
 * context's scratch: once a context has recorded, scratch that later calls outgrow is kept (not
 * freed) until swarm_destroy, so earlier graphs stay replayable; destroy graphs before their context.
 */
typedef struct swarm_graph swarm_graph;
swarm_status swarm_capture_begin(swarm_ctx* ctx);
swarm_status swarm_capture_end(swarm_ctx* ctx, swarm_graph** out);
swarm_status swarm_graph_launch(swarm_ctx* ctx, swarm_graph* graph);
swarm_status swarm_graph_destroy(swarm_graph* graph);

/*
 * Measurement aid (no part of the path): the rate this device reaches with a minimal kernel, to be
 * quoted next to the nominal peak a roofline is priced against.  Runs `reps` launches on the
 * context's stream, waits for them and returns the average rate in *out (host).
 *   SWARM_CAL_HBM_READ   streams `bytes` from buf with 16-byte loads           -> GB/s
 *   SWARM_CAL_HBM_WRITE  overwrites `bytes` of buf with 16-byte stores, one contiguous
 *                        4 KiB per workgroup in address order                   -> GB/s
 *   SWARM_CAL_MFMA_I8    register-resident loop of v_mfma_i32_32x32x32_i8, 16
 *                        independent accumulators per wave; buf >= 4 bytes     -> TOP/s
 *   SWARM_CAL_MFMA_FP4   the same with the 4-bit form of v_mfma_f32_32x32x64_f8f6f4, the
 *                        instruction the co-activation build runs on            -> TOP/s
 * buf: device, 16-byte aligned.  Choose bytes well above the 256 MB last-level cache to measure
 * memory, not cache.  Errors: SWARM_EINVAL for bad arguments or while recording a graph.
 */
typedef enum { SWARM_CAL_HBM_READ = 0, SWARM_CAL_HBM_WRITE = 1, SWARM_CAL_MFMA_I8 = 2, SWARM_CAL_MFMA_FP4 = 3 } swarm_calibration;
swarm_status swarm_calibrate(swarm_ctx* ctx, int32_t what, void* buf, size_t bytes, int32_t reps, double* out);

#ifdef __cplusplus
}
#endif
#endif /* SWARM_H_ */
