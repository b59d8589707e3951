// CPU oracle for the score -> select -> trace -> co-activation -> request-mapping path and the
// density pass over the co-activation counts.
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what each step of the
// path computes, written from the paper's definitions.  It shares no code with the HIP path
// and is only ever called from the tests, the smoke check and the benchmark's CPU-baseline
// leg.  The product path never routes through it.
//
// Every function takes host pointers.  `nthreads` splits *independent* output units (score
// rows, heads, row blocks of C, request groups) over std::thread workers; the arithmetic of a
// unit is the same whatever the thread count.
//
// Parity pins (tests/test_oracle_*.py): every function here is pinned by closed forms,
// special cases that reduce to numpy routines, hand-worked fixtures and invariants.  No
// function is "parity unpinned".
//
// Build: g++ -O2 -std=c++17 -shared -fPIC -pthread swarm_oracle.cpp -o liboracle.so

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <functional>
#include <thread>
#include <vector>

namespace {

// bf16 is the upper half of an IEEE binary32; widening is exact.
double bf16_to_double(uint16_t v) {
    uint32_t u = static_cast<uint32_t>(v) << 16;
    float f;
    std::memcpy(&f, &u, sizeof f);
    return static_cast<double>(f);
}

void parallel_for(int64_t n, int nthreads, const std::function<void(int64_t, int64_t)>& body) {
    if (nthreads <= 1 || n <= 1) { body(0, n); return; }
    int64_t nt = std::min<int64_t>(nthreads, n);
    std::vector<std::thread> pool;
    for (int64_t w = 0; w < nt; ++w) {
        int64_t lo = n * w / nt, hi = n * (w + 1) / nt;
        pool.emplace_back([&body, lo, hi] { body(lo, hi); });
    }
    for (auto& t : pool) t.join();
}

}  // namespace

extern "C" {

// ---------------------------------------------------------------------------------------
// Score (Section 2.3: relevance score of every KV entry against the query; inner products are
// the example the section names).
//
// kind 0, token keys  K[H][N][d]:      s = sum_c q_c * K_c
// kind 1, page summaries S[H][N][2][d] (channel-wise min then max of the page's keys):
//                                      s = sum_c max(q_c * mn_c, q_c * mx_c)
//   i.e. the channel-wise upper bound of q.key over any key inside the page's [min,max] box
//   (query-aware page selection, cited in Section 9; the formula is a reading, the paper gives none).
// Grouped-query attention: the G query heads that share KV head h add their scores.
// No 1/sqrt(d) scale: it is monotone and cannot change a top-k.
//
// q[B][H*G][d] bf16.  out_f32[B][H][N] = (float) of the double result.
// out_f64 (nullable) the double result; out_abs (nullable) = sum of |terms| (the magnitude the
// floating-point tolerance is scaled by).
// ---------------------------------------------------------------------------------------
// One entry's score against the G query heads of one KV head: s (fp64 sum, channels ascending, query
// heads in turn) and a (sum of the terms' magnitudes).
static void score_row(int kind, const uint16_t* row, const uint16_t* qhead, int G, int d, double* s_out, double* a_out) {
    double s = 0.0, a = 0.0;
    for (int g = 0; g < G; ++g) {
        const uint16_t* qv = qhead + (int64_t)g * d;
        for (int c = 0; c < d; ++c) {
            const double qc = bf16_to_double(qv[c]);
            double term;
            if (kind == 0) {
                term = qc * bf16_to_double(row[c]);
            } else {
                const double lo_t = qc * bf16_to_double(row[c]);       // q * min
                const double hi_t = qc * bf16_to_double(row[d + c]);   // q * max
                term = std::max(lo_t, hi_t);
            }
            s += term;
            a += std::fabs(term);
        }
    }
    *s_out = s;
    *a_out = a;
}

int oracle_score(int kind, const uint16_t* keys, const uint16_t* q, int B, int H, int G, int N, int d,
                 float* out_f32, double* out_f64, double* out_abs, int nthreads) {
    if (!keys || !q || B < 1 || H < 1 || G < 1 || N < 1 || d < 1 || (kind != 0 && kind != 1)) return -1;
    const int64_t row_len = (kind == 0) ? d : 2 * (int64_t)d;
    parallel_for((int64_t)B * H, nthreads, [&](int64_t lo, int64_t hi) {
        for (int64_t bh = lo; bh < hi; ++bh) {
            const int b = (int)(bh / H), h = (int)(bh % H);
            for (int n = 0; n < N; ++n) {
                double s, a;
                score_row(kind, keys + ((int64_t)h * N + n) * row_len, q + ((int64_t)b * H * G + (int64_t)h * G) * d, G, d, &s, &a);
                const int64_t o = ((int64_t)b * H + h) * N + n;
                if (out_f32) out_f32[o] = static_cast<float>(s);
                if (out_f64) out_f64[o] = s;
                if (out_abs) out_abs[o] = a;
            }
        }
    });
    return 0;
}

// The same scores for the listed entries only (medoid index, Section 5.2 Tier 1):
// out[b][h][m] = score of entry row_ids[h][m].  Returns -2 on an id outside [0,N).
int oracle_score_rows(int kind, const uint16_t* keys, const int32_t* row_ids, int M, const uint16_t* q, int B, int H, int G,
                      int N, int d, float* out_f32, double* out_f64, double* out_abs) {
    if (!keys || !row_ids || !q || B < 1 || H < 1 || G < 1 || N < 1 || M < 1 || d < 1 || (kind != 0 && kind != 1)) return -1;
    const int64_t row_len = (kind == 0) ? d : 2 * (int64_t)d;
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < H; ++h)
            for (int m = 0; m < M; ++m) {
                const int32_t n = row_ids[(int64_t)h * M + m];
                if (n < 0 || n >= N) return -2;
                double s, a;
                score_row(kind, keys + ((int64_t)h * N + n) * row_len, q + ((int64_t)b * H * G + (int64_t)h * G) * d, G, d, &s, &a);
                const int64_t o = ((int64_t)b * H + h) * M + m;
                if (out_f32) out_f32[o] = static_cast<float>(s);
                if (out_f64) out_f64[o] = s;
                if (out_abs) out_abs[o] = a;
            }
    return 0;
}

// ---------------------------------------------------------------------------------------
// Select (Section 2.3: keep the entries with the highest scores).  Per row of N float scores:
// order indices by (score descending, index ascending), take the first k, return them sorted
// by index.  -0 compares equal to +0 (IEEE), NaN ranks below every number.
// scores[rows][N] -> idx[rows][k].
// ---------------------------------------------------------------------------------------
int oracle_select(const float* scores, int64_t rows, int N, int k, int32_t* idx, int nthreads) {
    if (!scores || !idx || rows < 0 || N < 1 || k < 1 || k > N) return -1;
    parallel_for(rows, nthreads, [&](int64_t lo, int64_t hi) {
        std::vector<int32_t> order(N);
        for (int64_t r = lo; r < hi; ++r) {
            const float* s = scores + r * N;
            for (int i = 0; i < N; ++i) order[i] = i;
            std::stable_sort(order.begin(), order.end(), [s](int32_t a, int32_t b) {
                const bool na = std::isnan(s[a]), nb = std::isnan(s[b]);
                if (na || nb) return !na && nb;          // a number precedes a NaN; NaNs tie
                return s[a] > s[b];
            });
            std::vector<int32_t> top(order.begin(), order.begin() + k);
            std::sort(top.begin(), top.end());
            std::copy(top.begin(), top.end(), idx + r * k);
        }
    });
    return 0;
}

// ---------------------------------------------------------------------------------------
// Trace: binary activation matrix, one row per decode step (or per step x stream).
// idx[rows][H][k] -> A[H][rows][N] (uint8 0/1).  Returns -2 on an index outside [0,N).
// ---------------------------------------------------------------------------------------
int oracle_trace(const int32_t* idx, int64_t rows, int H, int k, int N, uint8_t* A) {
    if (!idx || !A || rows < 0 || H < 1 || k < 1 || N < 1) return -1;
    std::memset(A, 0, (size_t)H * rows * N);
    for (int64_t r = 0; r < rows; ++r)
        for (int h = 0; h < H; ++h)
            for (int j = 0; j < k; ++j) {
                const int32_t e = idx[(r * H + h) * k + j];
                if (e < 0 || e >= N) return -2;
                A[((int64_t)h * rows + r) * N + e] = 1;
            }
    return 0;
}

// ---------------------------------------------------------------------------------------
// Co-activation counts, the definition (Section 5.1, Step 1): element (i, j) is the number of
// rows of the trace in which entries i and j are both activated; the diagonal is an entry's
// own activation count.  A[rows][N] (0/1) -> C[N][N].  Triple loop; tiny inputs only.
// ---------------------------------------------------------------------------------------
int oracle_coact_dense(const uint8_t* A, int64_t rows, int N, int32_t* C) {
    if (!A || !C || rows < 0 || N < 1) return -1;
    for (int i = 0; i < N; ++i)
        for (int j = 0; j < N; ++j) {
            int64_t acc = 0;
            for (int64_t t = 0; t < rows; ++t) acc += (int64_t)A[t * N + i] * (int64_t)A[t * N + j];
            C[(int64_t)i * N + j] = (int32_t)acc;
        }
    return 0;
}

// ---------------------------------------------------------------------------------------
// Co-activation update from selections (same counts as above, k*k increments per row), with an
// optional fixed-point decay of the old matrix.  One call = one window:
//     C <- decay(C) + (counts of this window),
//     decay(c) = floor((c * decay_q16 + 2^15) / 2^16)   (round half up, Q16 multiplier),
//     decay_q16 = 65536 keeps C (plain accumulation), 0 discards it.
// New evidence enters undecayed.  The decay is not in the paper; it addresses the degradation of
// stale co-activation statistics the paper describes as its fourth challenge (Section 3.2).
// idx[rows][H][k], C[H][N][N] in/out.  Returns -2 on a bad index, -3 on a repeated index in a row,
// -5 when a count would pass INT32_MAX (counts are exact or the call fails; C is then partly updated).
// ---------------------------------------------------------------------------------------
int oracle_coact_update(const int32_t* idx, int64_t rows, int H, int k, int N, int32_t* C,
                        uint32_t decay_q16, int nthreads) {
    if (!idx || !C || rows < 0 || H < 1 || k < 1 || N < 1 || k > N || decay_q16 > 65536u) return -1;
    for (int64_t r = 0; r < rows * H; ++r) {
        std::vector<int32_t> v(idx + r * k, idx + (r + 1) * k);
        std::sort(v.begin(), v.end());
        if (v.front() < 0 || v.back() >= N) return -2;
        if (std::adjacent_find(v.begin(), v.end()) != v.end()) return -3;
    }
    // Row i of C[h] only depends on the trace rows that contain i: split (h, i) over workers.
    std::atomic<bool> overflow(false);
    parallel_for((int64_t)H * N, nthreads, [&](int64_t lo, int64_t hi) {
        if (decay_q16 != 65536u) {
            for (int64_t hi_row = lo; hi_row < hi; ++hi_row) {
                int32_t* crow = C + hi_row * N;
                for (int j = 0; j < N; ++j)
                    crow[j] = (int32_t)(((int64_t)crow[j] * (int64_t)decay_q16 + 32768) >> 16);
            }
        }
        for (int64_t r = 0; r < rows; ++r)
            for (int h = 0; h < H; ++h) {
                const int32_t* sel = idx + (r * H + h) * k;
                for (int a = 0; a < k; ++a) {
                    const int64_t hrow = (int64_t)h * N + sel[a];
                    if (hrow < lo || hrow >= hi) continue;
                    int32_t* crow = C + hrow * N;
                    for (int b = 0; b < k; ++b) {
                        if (crow[sel[b]] == INT32_MAX) { overflow.store(true); continue; }
                        ++crow[sel[b]];
                    }
                }
            }
    });
    return overflow.load() ? -5 : 0;
}

// ---------------------------------------------------------------------------------------
// A block of rows of the co-activation counts of one head (Section 5.1, Step 1, the same definition as
// above restricted to rows i in [r0, r1)): out[i - r0][j] = number of trace rows of head h that hold both
// i and j.  For matrices too large to keep whole on the host (65536 x 65536 counts are 16 GiB): the
// caller walks the matrix block by block.  idx[rows][H][k]; out[(r1 - r0)][N], overwritten.
// Returns -2 on a bad index, -3 on a repeated index in a row.
// ---------------------------------------------------------------------------------------
int oracle_coact_rows(const int32_t* idx, int64_t rows, int H, int k, int N, int h, int r0, int r1, int32_t* out,
                      int nthreads) {
    if (!idx || !out || rows < 0 || H < 1 || k < 1 || N < 1 || k > N || h < 0 || h >= H || r0 < 0 || r1 > N || r0 >= r1) return -1;
    for (int64_t r = 0; r < rows; ++r) {
        std::vector<int32_t> v(idx + (r * H + h) * k, idx + (r * H + h + 1) * k);
        std::sort(v.begin(), v.end());
        if (v.front() < 0 || v.back() >= N) return -2;
        if (std::adjacent_find(v.begin(), v.end()) != v.end()) return -3;
    }
    std::memset(out, 0, sizeof(int32_t) * (size_t)(r1 - r0) * N);
    // a row of the block only depends on the trace rows that contain it: split the block's rows over workers
    parallel_for(r1 - r0, nthreads, [&](int64_t lo, int64_t hi) {
        for (int64_t r = 0; r < rows; ++r) {
            const int32_t* sel = idx + (r * H + h) * k;
            for (int a = 0; a < k; ++a) {
                const int64_t i = (int64_t)sel[a] - r0;
                if (i < lo || i >= hi) continue;
                int32_t* crow = out + i * N;
                for (int b = 0; b < k; ++b) ++crow[sel[b]];
            }
        }
    });
    return 0;
}

// ---------------------------------------------------------------------------------------
// Request mapping (Section 6.1: merge of the activated clusters with the DRAM-resident ones
// filtered out, then decoupled entry-bucket scheduling).  Per group g (head = g % H):
//   1. clusters = { e2c[head][e] : e in sel[g] } minus those whose bit is set in `resident`;
//   2. visit them in ascending (replication factor, cluster id); the replication factor is the
//      number of non-negative slots in replicas[cluster][0..R);
//   3. a cluster goes to the candidate SSD whose bucket load is smallest (ties: smallest SSD
//      id); the bucket load grows by weight[cluster] (1 when weight is null);
//   4. queues are emitted SSD-major in insertion order: q_off[g][D+1], q_cluster[g][cap],
//      q_load[g][D].
// The unit routed is a cluster (the paper's atomic retrieval unit); with Nc = N, identity e2c
// and unit weights this is exactly the paper's per-entry rule.
// An entry id of -1 is padding (ragged selections) and is skipped.
// Returns -2 on any other out-of-range entry / cluster / SSD id, -4 if cap is too small.
// ---------------------------------------------------------------------------------------
int oracle_map(const int32_t* sel, int64_t groups, int S, int H, int N, const int32_t* e2c, int Nc,
               const int32_t* replicas, int R, int D, const int32_t* weight, const uint32_t* resident,
               int32_t* q_off, int32_t* q_cluster, int32_t* q_load, int cap, int nthreads) {
    if (!sel || !e2c || !replicas || !q_off || !q_cluster || !q_load) return -1;
    if (groups < 0 || S < 1 || H < 1 || N < 1 || Nc < 1 || R < 1 || D < 1 || R > D || cap < 1) return -1;
    std::vector<int> status((size_t)std::max<int64_t>(groups, 1), 0);
    parallel_for(groups, nthreads, [&](int64_t lo, int64_t hi) {
        for (int64_t g = lo; g < hi; ++g) {
            const int h = (int)(g % H);
            std::vector<uint8_t> seen(Nc, 0);
            for (int s = 0; s < S; ++s) {
                const int32_t e = sel[g * S + s];
                if (e == -1) continue;                            // padding of a ragged selection
                if (e < 0 || e >= N) { status[g] = -2; break; }
                const int32_t c = e2c[(int64_t)h * N + e];
                if (c < 0 || c >= Nc) { status[g] = -2; break; }
                seen[c] = 1;
            }
            if (status[g]) continue;
            struct Item { int rf; int32_t c; };
            std::vector<Item> items;
            for (int32_t c = 0; c < Nc; ++c) {
                if (!seen[c]) continue;
                const int64_t gc = (int64_t)h * Nc + c;
                if (resident && ((resident[gc >> 5] >> (gc & 31)) & 1u)) continue;
                int rf = 0;
                for (int r = 0; r < R; ++r) {
                    const int32_t dsk = replicas[gc * R + r];
                    if (dsk >= D) status[g] = -2;
                    if (dsk >= 0) ++rf;
                }
                if (rf == 0) status[g] = -2;
                items.push_back({rf, c});
            }
            if (status[g]) continue;
            if ((int)items.size() > cap) { status[g] = -4; continue; }
            std::stable_sort(items.begin(), items.end(),
                             [](const Item& a, const Item& b) { return a.rf < b.rf; });
            std::vector<int64_t> load(D, 0);
            std::vector<std::vector<int32_t>> bucket(D);
            for (const Item& it : items) {
                const int64_t gc = (int64_t)h * Nc + it.c;
                int best = -1;
                for (int r = 0; r < R; ++r) {
                    const int32_t dsk = replicas[gc * R + r];
                    if (dsk < 0) continue;
                    if (best < 0 || load[dsk] < load[best] || (load[dsk] == load[best] && dsk < best)) best = dsk;
                }
                bucket[best].push_back(it.c);
                load[best] += weight ? weight[gc] : 1;
            }
            int32_t pos = 0;
            for (int dsk = 0; dsk < D; ++dsk) {
                q_off[g * (D + 1) + dsk] = pos;
                for (int32_t c : bucket[dsk]) q_cluster[g * cap + pos++] = c;
                q_load[g * D + dsk] = (int32_t)load[dsk];
            }
            q_off[g * (D + 1) + D] = pos;
            for (int32_t p = pos; p < cap; ++p) q_cluster[g * cap + p] = -1;
        }
    });
    for (int64_t g = 0; g < groups; ++g)
        if (status[g]) return status[g];
    return 0;
}

// ---------------------------------------------------------------------------------------
// Medoid-indexed retrieval (Section 5.2, Tier 1: every cluster's medoid is its index entry, scored
// against the query to decide whether the cluster is retrieved; Section 6.1: the activated clusters
// are merged into the set of entries to transfer).
//
// oracle_score_rows: the score of oracle_score, for the listed entries only:
//   out[b][h][m] = score of entry row_ids[h][m]   (fp32 and fp64; abs = sum of |terms|)
// oracle_expand_clusters: per group g (head g % H), the distinct activated clusters in ascending id,
// each replaced by its member entries in stored order: entries[g][0..count[g]) then -1 padding.
// Entries shared by several clusters appear once per cluster; the merge into a set (and the removal
// of DRAM-resident entries) is the mapping step's.  clusters int32 [groups][Sc] (-1 = padding);
// cl_off int32 [H][Nc+1] offsets into cl_entries int32 [H][E].  Returns -4 if cap_e is too small.
// ---------------------------------------------------------------------------------------
int oracle_expand_clusters(const int32_t* clusters, int64_t groups, int Sc, int H, int Nc, const int32_t* cl_off,
                           const int32_t* cl_entries, int E, int32_t* entries, int32_t* count, int cap_e) {
    if (!clusters || !cl_off || !cl_entries || !entries || !count || groups < 0 || Sc < 1 || H < 1 || Nc < 1 || cap_e < 1) return -1;
    for (int64_t g = 0; g < groups; ++g) {
        const int h = (int)(g % H);
        std::vector<uint8_t> seen(Nc, 0);
        for (int s = 0; s < Sc; ++s) {
            const int32_t c = clusters[g * Sc + s];
            if (c == -1) continue;
            if (c < 0 || c >= Nc) return -2;
            seen[c] = 1;
        }
        int32_t n = 0;
        for (int c = 0; c < Nc; ++c) {
            if (!seen[c]) continue;
            const int32_t lo = cl_off[(int64_t)h * (Nc + 1) + c], hi = cl_off[(int64_t)h * (Nc + 1) + c + 1];
            if (lo < 0 || hi < lo || hi > E) return -2;
            for (int32_t p = lo; p < hi; ++p) {
                if (n >= cap_e) return -4;
                entries[g * cap_e + n++] = cl_entries[(int64_t)h * E + p];
            }
        }
        count[g] = n;
        for (int32_t p = n; p < cap_e; ++p) entries[g * cap_e + p] = -1;
    }
    return 0;
}

// ---------------------------------------------------------------------------------------
// Submission order (Section 6.1, last paragraph: the head entry of every bucket is taken in turn and
// the heads form one submission batch).  From the buckets of oracle_map: order[g] lists the routed
// items batch by batch -- batch b holds the b-th item of every bucket that has one, in ascending SSD
// id -- and batch_off[g][b] is where batch b starts (batch_off[g][nb[g]] = number of items).
// order int32 [groups][cap] (-1 padded); batch_off int32 [groups][cap+1] (entries past nb[g] repeat
// the total); nb int32 [groups].
// ---------------------------------------------------------------------------------------
int oracle_submission_order(const int32_t* q_off, const int32_t* q_cluster, int64_t groups, int D, int cap, int32_t* order,
                            int32_t* batch_off, int32_t* nb) {
    if (!q_off || !q_cluster || !order || !batch_off || !nb || groups < 0 || D < 1 || cap < 1) return -1;
    for (int64_t g = 0; g < groups; ++g) {
        const int32_t* off = q_off + g * (D + 1);
        std::vector<int32_t> head(off, off + D);                   // next unread position of every bucket
        int32_t n = 0, b = 0;
        for (;;) {
            bool any = false;
            const int32_t start = n;
            for (int d = 0; d < D; ++d)
                if (head[d] < off[d + 1]) { order[g * cap + n++] = q_cluster[g * cap + head[d]++]; any = true; }
            if (!any) break;
            batch_off[g * (cap + 1) + b++] = start;
        }
        nb[g] = b;
        for (int32_t p = b; p <= cap; ++p) batch_off[g * (cap + 1) + p] = n;
        for (int32_t p = n; p < cap; ++p) order[g * cap + p] = -1;
    }
    return 0;
}

int oracle_hardware_threads(void) { return (int)std::thread::hardware_concurrency(); }

// ---------------------------------------------------------------------------------------
// Co-activation density and medoid queue (Section 5.1: the probability equation of Step 1, the
// distance of Step 2, and the density loop and the descending sort of Algorithm 1's Step 3).
//
//   total   = sum over all (k, l) of C[k][l]                       (the denominator of P)
//   P(i,j)  = C[i][j] / total ;  d(i,j) = 1 - P(i,j)               (fp64, each operation rounded once)
//   rho[i]  = number of j with d(i,j) <= tau                       (Algorithm 1: every j, "<=")
//             flags bit 0: leave out j = i, bit 1: "<" instead of "<="  (the density equation's form)
//   queue   = entries in descending rho, equal rho in ascending entry id (the paper does not order ties)
// total = 0 leaves P undefined; no pair is then counted.  totals_in (nullable) replaces the computed
// denominator, e.g. to rescale.  C int32 [H][N][N]; rho int32 [H][N]; queue int32 [H][N];
// totals_out int64 [H].
// ---------------------------------------------------------------------------------------
int oracle_density(const int32_t* C, int H, int N, const int64_t* totals_in, double tau, uint32_t flags, int32_t* rho,
                   int32_t* queue, int64_t* totals_out, int nthreads) {
    if (!C || !rho || !queue || !totals_out || H < 1 || N < 1) return 1;
    const bool skip_self = flags & 1u, strict = flags & 2u;
    for (int h = 0; h < H; ++h) {
        const int32_t* Ch = C + (size_t)h * N * N;
        int64_t total = 0;
        for (size_t e = 0; e < (size_t)N * N; ++e) total += Ch[e];
        if (totals_in) total = totals_in[h];
        totals_out[h] = total;
        int32_t* rh = rho + (size_t)h * N;
        parallel_for(N, nthreads, [&](int64_t lo, int64_t hi) {
            for (int64_t i = lo; i < hi; ++i) {
                int32_t count = 0;
                for (int j = 0; j < N; ++j) {
                    if (skip_self && j == i) continue;
                    if (total == 0) continue;
                    const double P = static_cast<double>(Ch[(size_t)i * N + j]) / static_cast<double>(total);
                    const double d = 1.0 - P;
                    if (strict ? (d < tau) : (d <= tau)) ++count;
                }
                rh[i] = count;
            }
        });
        std::vector<int32_t> ids(N);
        for (int i = 0; i < N; ++i) ids[i] = i;
        std::stable_sort(ids.begin(), ids.end(), [&](int32_t a, int32_t b) { return rh[a] > rh[b]; });
        std::memcpy(queue + (size_t)h * N, ids.data(), sizeof(int32_t) * N);
    }
    return 0;
}

// ---------------------------------------------------------------------------------------
// Cluster maintenance over the local window (Section 6.2, the distance between a newly generated
// entry and a cluster): for every new entry e and every cluster i with medoid m_i,
//   f(e, m_i) = number of the window's W steps in which e and m_i are both activated,
//   d(e, C_i) = 1 - f(e, m_i) / W                                          (fp64)
// and e joins every cluster with d < tau.  A joining entry is placed on the cluster's next SSD:
// disk = (id_i + |C_i| + 1) mod D, where |C_i| grows by one with every entry that joins (new entries
// are taken in the order given: a reading, the paper places one entry at a time).
// sel int32 [W][H][k]; new_ids int32 [H][n_new]; medoids int32 [H][Nc]; primary, size int32 [H][Nc]
// (nullable together: no placement); f_out int32 [H][n_new][Nc]; member uint8 [H][n_new][Nc];
// disk int32 [H][n_new][Nc] (-1 where not joined; nullable).
// ---------------------------------------------------------------------------------------
int oracle_window_assign(const int32_t* sel, int W, int H, int k, int N, const int32_t* new_ids, int n_new,
                         const int32_t* medoids, int Nc, double tau, const int32_t* primary, const int32_t* size, int D,
                         int32_t* f_out, uint8_t* member, int32_t* disk) {
    if (!sel || !new_ids || !medoids || !f_out || !member || W < 1 || H < 1 || k < 1 || n_new < 1 || Nc < 1) return 1;
    if ((primary == nullptr) != (size == nullptr) || (disk && (!primary || D < 1))) return 1;
    std::vector<uint8_t> act((size_t)W * N);
    for (int h = 0; h < H; ++h) {
        std::fill(act.begin(), act.end(), 0);
        for (int t = 0; t < W; ++t)
            for (int j = 0; j < k; ++j) {
                const int32_t e = sel[((size_t)t * H + h) * k + j];
                if (e >= 0 && e < N) act[(size_t)t * N + e] = 1;
            }
        std::vector<int32_t> grown(Nc, 0);
        for (int a = 0; a < n_new; ++a) {
            const int32_t e = new_ids[(size_t)h * n_new + a];
            for (int c = 0; c < Nc; ++c) {
                const int32_t m = medoids[(size_t)h * Nc + c];
                int32_t f = 0;
                if (e >= 0 && e < N && m >= 0 && m < N)
                    for (int t = 0; t < W; ++t) f += act[(size_t)t * N + e] & act[(size_t)t * N + m];
                const double d = 1.0 - static_cast<double>(f) / static_cast<double>(W);
                const bool join = d < tau;
                const size_t o = ((size_t)h * n_new + a) * Nc + c;
                f_out[o] = f;
                member[o] = join;
                if (disk) {
                    disk[o] = -1;
                    if (join) {
                        const int64_t sz = (int64_t)size[(size_t)h * Nc + c] + grown[c];
                        disk[o] = (int32_t)(((int64_t)primary[(size_t)h * Nc + c] + sz + 1) % D);
                        ++grown[c];
                    }
                }
            }
        }
    }
    return 0;
}

}  // extern "C"
