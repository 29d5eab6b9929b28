/*
 * quiver.h -- C ABI of the MI355X (gfx950) library for the QuIVer query hot path
 * (arxiv 2605.02171): 2-bit Sign-Magnitude encoding, beam search over a fixed-degree
 * graph in code space, float32 cosine rerank.
 *
 * Conventions for every call
 *   - "device pointer" = memory on the current HIP device, allocated and owned by the
 *     caller (the Python binding passes torch tensors' data_ptr()).  The library borrows
 *     buffers; it never frees or reallocates them.  The caller keeps them alive until the
 *     work queued on `stream` has completed.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All device
 *     work is queued on it and the call returns without waiting, unless stated otherwise.
 *   - Return value: 0 (QV_OK) or a negative QV_ERR_* code.  Argument errors are found on
 *     the host before anything is launched; nothing is written in that case.
 *   - ids are uint32; 0xFFFFFFFF (QV_EMPTY) marks "no node".
 */
#ifndef QUIVER_H
#define QUIVER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define QV_EMPTY 0xFFFFFFFFu

#define QV_OK 0
#define QV_ERR_INVALID_ARG (-1) /* a size or count is out of range                     */
#define QV_ERR_NULL (-2)        /* a required pointer is NULL                          */
#define QV_ERR_DIM (-3)         /* d < 1 or d > QV_MAX_DIM                             */
#define QV_ERR_EF_LT_K (-4)     /* k > ef: the rerank can only return list members     */
#define QV_ERR_EF_RANGE (-5)    /* ef < 1 or ef > QV_MAX_EF                            */
#define QV_ERR_WORKSPACE (-6)   /* workspace NULL, misaligned or too small             */
#define QV_ERR_HIP (-7)         /* a HIP runtime call failed (see qv_last_hip_error)   */
#define QV_ERR_NOMEM (-8)       /* host allocation failed                              */
#define QV_ERR_UNSUPPORTED (-9) /* the shape is outside what this entry point handles */
#define QV_ERR_SCRATCH_LIMIT (-10) /* qv_search_static: the batch needs more than QV_STATIC_SCRATCH_BYTES */

#define QV_MAX_DIM 65536
#define QV_MAX_EF 1024
#define QV_MAX_DEGREE 4096
#define QV_MAX_SCAN_K 64

/* bits of the per-vector / per-query status words */
#define QV_STATUS_NONFINITE 1u      /* encode: the vector holds Inf/NaN, its code is unspecified;           */
                                    /* search: the query holds Inf/NaN and was not searched                 */
#define QV_STATUS_VISITED_FULL 2u   /* search: the on-chip visited table filled up; results stay exact,     */
                                    /* n_dist_evals may count some nodes more than once                     */
#define QV_STATUS_BAD_EDGE 4u       /* search: an adjacency entry >= n was skipped                          */
#define QV_STATUS_TIMEOUT 8u        /* search: Stage 2 in other waves gave up waiting for the list (empty result) */

/* Words (uint64) per code: 2 * ceil(d / 64); 0 if d is out of range.  Host only. */
int qv_code_words(int d);

/*
 * 1. Encode (paper Sec. 3.1, encoding equations): tau = mean_i |x_i| (exact mean),
 *    pos_i = [x_i > 0], strong_i = [|x_i| > tau].
 *    x      device, [n][d] float32 row-major.
 *    codes  device, [n][qv_code_words(d)] uint64: W = ceil(d/64) words of sign bits, then W
 *           words of magnitude bits; dimension i is bit i%64 (bit 0 = LSB) of word i/64; bits
 *           of dimensions >= d are 0.
 *    status device, [n] uint32 or NULL: receives QV_STATUS_NONFINITE or 0 per vector.
 *    0 <= n <= 2^32 (QV_ERR_INVALID_ARG otherwise; n = 0 does nothing).  Asynchronous on `stream`.
 */
int qv_encode(const float* x, int64_t n, int d, uint64_t* codes, uint32_t* status, void* stream);

/*
 * Test aid (paper Sec. 3.1, Table 1): symmetric distance for pairs of codes,
 *    out[p] = sum over dimensions with differing sign bits of (1+strong_a)(1+strong_b).
 *    codes_a/codes_b device code arrays as written by qv_encode; ia/ib device int64 [npairs]
 *    row indices (the caller guarantees they are in range); out device uint32 [npairs].
 */
int qv_bq_distance(const uint64_t* codes_a, const int64_t* ia, const uint64_t* codes_b, const int64_t* ib,
                   int64_t npairs, int d, uint32_t* out, void* stream);

/*
 * Measurement aid (paper Sec. 4.2, "Cache friendliness": a hop touches one code of D/4 bytes): reads the
 * code rows ids[0 .. n_ids) (device uint32, each < n -- the caller guarantees it; n_ids is used in
 * multiples of 64) with the search kernel's gather pattern and no arithmetic, to measure the rate the
 * memory system sustains for that pattern.  sink: device uint64[1], scratch.
 */
int qv_gather_probe(const uint64_t* codes, int64_t n, int d, const uint32_t* ids, int64_t n_ids, uint64_t* sink,
                    void* stream);

/*
 * 2. Load (paper Sec. 4.2: hot data = codes + flat adjacency, cold data = float32 vectors).
 *    Creates a host-side handle that remembers the borrowed device buffers; copies nothing.
 *    adj    device, [n][R] uint32, QV_EMPTY = empty slot (rows need not be packed to the left)
 *    codes  device, [n][qv_code_words(d)] uint64 in qv_encode's layout (or another layout: qv_index_set_code_layout)
 *    vecs   [n][d] float32, only read by the rerank: device memory, or host memory the device can address
 *           (hipHostMalloc / pinned): the paper's cold store then stays in host RAM and the rerank's ef rows per
 *           query travel over PCIe
 *    entry  node every search starts from, < n
 *    The call asks the runtime once where `vecs` lives (device or host memory): the rerank runs inside the search
 *    kernel only over device memory (qv_index_set_tuning).
 *    1 <= R <= QV_MAX_DEGREE, 1 <= n < 2^32 - 1.
 */
typedef struct qv_index qv_index;
int qv_index_load(qv_index** out, int64_t n, int d, int R, const uint32_t* adj, const uint64_t* codes,
                  const float* vecs, uint32_t entry);
void qv_index_free(qv_index* index); /* frees the handle only; NULL is allowed */

/* Optional per-query outputs of qv_search; every pointer is a device pointer or NULL. */
typedef struct qv_trace {
    uint32_t* cand_ids;     /* [nq][ef]  final list, sorted by (distance, id); QV_EMPTY padded          */
    uint32_t* cand_dist;    /* [nq][ef]  their code-space distances; QV_EMPTY padded                    */
    uint32_t* n_cand;       /* [nq]      length of the final list                                       */
    uint32_t* n_expanded;   /* [nq]      nodes expanded                                                 */
    uint32_t* n_dist_evals; /* [nq]      code-space distances computed                                  */
    uint32_t* visit_order;  /* [nq][visit_cap] ids in the order they were expanded; QV_EMPTY padded     */
    int64_t visit_cap;      /*           entries per query in visit_order (0 if unused)                 */
    uint32_t* status;       /* [nq]      QV_STATUS_* bits                                               */
} qv_trace;

/* Bytes of device scratch qv_search needs for this shape (0 on invalid arguments).  Host only. */
size_t qv_search_workspace_bytes(int64_t nq, int d, int k, int ef);

/*
 * 3. Search (paper Sec. 3.3): per query, encode it once (Stage 1 preamble), run the greedy
 *    best-first beam search with an ef-wide list keyed by (code distance, id) from the index's
 *    entry node, then (Stage 2) score every list member with the exact cosine similarity to the
 *    float32 query and return the best k by (score descending, id ascending).
 *    queries   device, [nq][d] float32
 *    ids       device, [nq][k] uint32, QV_EMPTY where the list was shorter than k
 *    scores    device, [nq][k] float32 cosine (accumulated in double, rounded once), -inf padded;
 *              a zero-norm query or vector scores 0
 *    workspace device, 256-byte aligned, >= qv_search_workspace_bytes(nq, d, k, ef); contents
 *              are scratch (concurrent searches need separate workspaces)
 *    trace     NULL or a struct of optional outputs
 *    1 <= k <= ef <= QV_MAX_EF.  nq == 0 is allowed and does nothing.
 *    Non-finite input (a precondition violation, reported and never silent): a query that holds Inf or NaN is not
 *    searched -- all k of its ids are QV_EMPTY and its scores -inf, its list is empty (n_cand, n_expanded,
 *    n_dist_evals 0; cand_ids, cand_dist, visit_order QV_EMPTY) and its trace status is QV_STATUS_NONFINITE; the other
 *    queries of the batch are unaffected.  A list member whose stored vector holds Inf or NaN scores -inf, i.e. it
 *    ranks after every finite score (by id among such members).
 */
int qv_search(const qv_index* index, const float* queries, int64_t nq, int k, int ef, uint32_t* ids, float* scores,
              void* workspace, size_t workspace_bytes, const qv_trace* trace, void* stream);

/*
 * qv_search for callers that cannot allocate device memory or hand over a workspace: code running under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and same results as
 * qv_search, but the scratch memory is a buffer of QV_STATIC_SCRATCH_BYTES that is part of the library's device code
 * (one per GPU, held until the process ends); the call allocates and frees nothing.
 *    - A batch whose qv_search_workspace_bytes(nq, d, k, ef) exceeds QV_STATIC_SCRATCH_BYTES is refused with
 *      QV_ERR_SCRATCH_LIMIT before anything is launched (16 MiB hold 10,000 queries of 768 dimensions at ef = 64, or
 *      1,700 at ef = 1024); split larger batches or use qv_search.
 *    - All calls on one GPU share that GPU's buffer: calls that overlap in time on the same GPU (two streams, two
 *      threads) race on it and must not be made; calls on one stream, or ordered by events, are fine.
 *    - The buffer keeps the previous call's contents; every part a call reads it has written first, so nothing
 *      needs clearing between calls.
 *    - More than 64 GPUs in one process: QV_ERR_UNSUPPORTED for device numbers from 64 on.
 */
#define QV_STATIC_SCRATCH_BYTES (16u << 20)
int qv_search_static(const qv_index* index, const float* queries, int64_t nq, int k, int ef, uint32_t* ids,
                     float* scores, const qv_trace* trace, void* stream);

/*
 * Stage timer: when one is attached, every qv_search on that index records HIP events around its
 * three stages (query encode together with the launch-order pass, the beam search kernel, rerank) on the
 * search's stream.  qv_timer_read waits for the recorded events and returns milliseconds per stage per
 * recorded call.  When the rerank runs inside the search kernel (qv_index_rerank_fused), the second stage holds
 * both and the third is the gap between two event records.
 */
typedef struct qv_timer qv_timer;
int qv_timer_create(qv_timer** out, int max_calls);
void qv_timer_free(qv_timer* t);
void qv_index_set_timer(qv_index* index, qv_timer* t /* NULL detaches */);
/* ms: host float [max_calls][3]; returns the number of recorded calls (>= 0) or an error; resets the timer */
int qv_timer_read(qv_timer* t, float* ms, int max_calls);

/*
 * Brute-force scan in code space and overlap probe (paper Sec. 6, "Practical compatibility test": compare
 * the code-ranked top K with the float32-ranked top K on a sample before building an index; Sec. 5.5,
 * Table 10 reports the same "Top-10 overlap").
 *    qv_bq_scan: for every query code the K base codes with the smallest (distance, id).
 *       codes   device, [n][qv_code_words(d)];  qcodes device, [nq][qv_code_words(d)] (qv_encode's layout)
 *       ids, dist device uint32 [nq][K], sorted by (distance, id), QV_EMPTY padded when n < K
 *       workspace device, 256-byte aligned, >= qv_bq_scan_workspace_bytes(n, nq, K)
 *       1 <= K <= QV_MAX_SCAN_K.
 *    qv_topk_overlap: hits[q] = number of entries of a[q][0..K) that occur in b[q][0..K) (device uint32
 *       arrays [nq][K]; QV_EMPTY never matches); the probe's figure is sum(hits) / (nq * K).
 */
size_t qv_bq_scan_workspace_bytes(int64_t n, int64_t nq, int K);
int qv_bq_scan(const uint64_t* codes, int64_t n, int d, const uint64_t* qcodes, int64_t nq, int K, uint32_t* ids,
               uint32_t* dist, void* workspace, size_t workspace_bytes, void* stream);
int qv_topk_overlap(const uint32_t* a, const uint32_t* b, int64_t nq, int K, uint32_t* hits, void* stream);

/*
 * Graph construction in code space (paper Sec. 3.2, Algorithm 1 "BQ-Vamana Edge Selection": candidates
 * sorted by distance to the target t, c is kept iff dist(c,t) <= alpha * dist(c,s) for every s kept before
 * it, at most R kept; Sec. 2.2: when t selects b, t becomes a candidate of b and b's row is re-selected).
 * Batch-synchronous reading (the paper's lock-based concurrent insertion, Sec. 4.1, has no single defined
 * result): nodes enter in id order in batches of max(1, done/50) (at most max_batch); every node of a
 * batch searches the graph as it stood before the batch (beam width L from `entry`) and selects its
 * out-edges from its final list plus its current out-neighbours; then every selected node takes the
 * selecting nodes (at most the 192 nearest per batch) into its row if they fit and re-selects the row
 * from (old row U new candidates) otherwise.  The order of ids inside a row carries no meaning.
 *    codes   device, [n][qv_code_words(d)]         adj  device, [n][R] uint32, written in full
 *    1 <= R <= 64, 1 <= L <= 192, alpha >= 1, entry < n; d <= 1536 (planes of up to 24 words: the selection
 *    kernels keep a whole code in registers; wider: QV_ERR_UNSUPPORTED).  The kernels are compiled for planes of
 *    2, 4, 6, 8, 12, 16 and 24 words; codes of another width are copied into the workspace with zero words
 *    appended to every plane (n more rows of the next compiled width), which changes no distance.
 *    workspace device, 256-byte aligned, >= qv_build_workspace_bytes(n, d, R, L, max_batch) (8 bytes per node for grouping
 *              a batch's new edges by target, plus the lists of the largest batch)
 *    max_batch >= 1; the largest batch, min(max(1, n / 50), max_batch) nodes, times R must stay below 2^31
 *    (QV_ERR_INVALID_ARG otherwise: lower max_batch).
 * All work is queued on `stream`; the call returns when everything is queued.
 */
size_t qv_build_workspace_bytes(int64_t n, int d, int R, int L, int64_t max_batch);   /* 0: arguments out of range */
int qv_build_graph(const uint64_t* codes, int64_t n, int d, int R, int L, double alpha, uint32_t entry,
                   int64_t max_batch, uint32_t* adj, void* workspace, size_t workspace_bytes, void* stream);

/*
 * The two alternative encodings of the paper's ablation (Sec. 5.5 "Encoding Ablation", Table 10), through the
 * same path.  Every *_enc call is its namesake above with an `encoding` argument; QV_ENC_SM is the method itself.
 *    QV_ENC_SIGN1  "1-bit sign": the sign plane alone, qv_code_words_enc(d) = ceil(d/64) words per vector;
 *                  distance = number of differing signs.
 *    QV_ENC_SQ2    "2-bit SQ": every dimension falls into one of four equal-width buckets, distance = sum of
 *                  |level_a - level_b| (L1).  The paper names no range; here it is [-2 tau, +2 tau] with tau the
 *                  vector's exact mean magnitude (edges at -tau, 0, +tau; values beyond the range fall into the
 *                  outer buckets), the range with which the quantiser ranks as Table 10 reports it: level 3 iff
 *                  x > tau, 2 iff 0 < x <= tau, 1 iff -tau <= x <= 0, 0 iff x < -tau.  Two bit-planes, low bit of
 *                  the level first, packed like the Sign-Magnitude planes.
 * qv_index_set_encoding tells an index which encoding its `codes` are in (queries are then encoded the same way).
 * Widths: encode, distance, scan and search take any d (the search kernel is compiled for the same plane widths in all
 * three encodings; at widths other than 768-d the ablation encodings use the default number of lanes per row whatever
 * qv_index_set_tuning says); qv_build_graph_enc takes d <= 1536 like qv_build_graph; its workspace is
 * qv_build_workspace_bytes_enc.  An unknown encoding is QV_ERR_INVALID_ARG (0 words from qv_code_words_enc).
 */
#define QV_ENC_SM 0
#define QV_ENC_SIGN1 1
#define QV_ENC_SQ2 2
int qv_code_words_enc(int d, int encoding);
int qv_encode_enc(const float* x, int64_t n, int d, int encoding, uint64_t* codes, uint32_t* status, void* stream);
int qv_bq_distance_enc(const uint64_t* codes_a, const int64_t* ia, const uint64_t* codes_b, const int64_t* ib,
                       int64_t npairs, int d, int encoding, uint32_t* out, void* stream);
int qv_bq_scan_enc(const uint64_t* codes, int64_t n, int d, int encoding, const uint64_t* qcodes, int64_t nq, int K,
                   uint32_t* ids, uint32_t* dist, void* workspace, size_t workspace_bytes, void* stream);
size_t qv_build_workspace_bytes_enc(int64_t n, int d, int encoding, int R, int L, int64_t max_batch);
int qv_build_graph_enc(const uint64_t* codes, int64_t n, int d, int encoding, int R, int L, double alpha, uint32_t entry,
                       int64_t max_batch, uint32_t* adj, void* workspace, size_t workspace_bytes, void* stream);
int qv_index_set_encoding(qv_index* index, int encoding);

/* Tunables of the search kernel (defaults picked from the shape when 0).  Host only.
 *    visited_slots   slots of the per-query visited table, 1024..28672 (rounded up to a multiple of 1024; to a
 *                    power of two and at most 8192 with 32-bit entries; as a cache of 16-bit entries every eighth
 *                    slot is a counter, so 7/8 of the slots hold ids)
 *    lanes_per_row   lanes that share one neighbour's code during the gather (1, 2, 4, 8 or 16)
 *    table_format    0: 16-bit visited-table entries whenever the graph is small enough for them, else 32-bit;
 *                    32: always 32-bit entries
 *    visited_mode    how the per-query visited set of Sec. 4.1 is kept (the final lists, their order and the
 *                    expansion order are the same in both modes; only the number of distance evaluations differs):
 *                    QV_VISITED_EXACT  never forgets an id; when the table is nearly full it stops taking ids
 *                    QV_VISITED_CACHE  a small table in which new ids displace old ones: a forgotten node that
 *                                      comes up again is evaluated again and dropped when it is merged
 *                    Either way status bit 2 of a query says that nodes may have been evaluated more than once.
 *    rerank_mode     where Stage 2 of Sec. 3.3 runs (same scores to the tolerance of the rerank, same order):
 *                    QV_RERANK_SEPARATE  a kernel of its own after the search.
 *                    QV_RERANK_FUSED     inside the search kernel, by the wave that finished the query's Stage 1, so
 *                                        that its row reads fill the time other waves spend waiting for gathers.
 *                    QV_RERANK_TAIL      inside the search kernel, by other waves: the launch holds one more workgroup
 *                                        per query, which starts when the last searches are under way, waits for its
 *                                        query's list if need be (the search it waits for is always running by then)
 *                                        and scores it, so that Stage 2 fills the memory system the emptier end of
 *                                        the batch leaves idle.  A wait that does not end within seconds (never seen)
 *                                        is reported as status bit QV_STATUS_TIMEOUT with an empty result.
 *                    The two in-kernel forms apply to ef <= 128 and vectors in device memory; elsewhere the stage runs
 *                    as a kernel of its own.
 *                    0: QV_RERANK_TAIL wherever it applies (the fastest form at every width measured). */
#define QV_VISITED_EXACT 1
#define QV_VISITED_CACHE 2
#define QV_RERANK_SEPARATE 1
#define QV_RERANK_FUSED 2
#define QV_RERANK_TAIL 3
int qv_index_set_tuning(qv_index* index, int visited_slots, int lanes_per_row, int table_format, int visited_mode,
                        int rerank_mode);
/* 1 if a search with this beam width runs Stage 2 inside the search kernel as the index is set up now, else 0
 * (QV_ERR_NULL without an index).  Host only. */
int qv_index_rerank_fused(const qv_index* index, int ef);

/*
 * Layout of an index's codes (an option of this library, not of the paper; Sec. 4.2 fixes only what the hot data
 * holds).  Two things cost the search time without changing what it computes, and both are a matter of where the
 * words of a code row sit:
 *   - the search kernel is compiled for certain plane widths (2, 4, 6, 8, 12, 16, 24, 32, 48 words of 64 bits for
 *     Sign-Magnitude codes); other widths (960-d = 15 words, 300-d = 5 words, ...) run a general kernel that is
 *     about 1.7x slower.  Planes padded with zero words to the next compiled width take the fast kernel, and
 *     zero words add nothing to any distance;
 *   - the memory system moves 128-byte lines and rows are gathered at random: a 96-byte row (384-d) stored
 *     densely straddles a line boundary every other time.  Rows stored `stride` words apart, stride * 8 a
 *     divisor or a multiple of 128, touch the fewest lines there are.
 * A layout is (plane_words, stride): row i starts at word i * stride; its plane p occupies words
 * [p * plane_words, p * plane_words + ceil(d/64)) of the row and is followed by zero words up to plane_words.
 *   qv_code_layout   (host only) the layout recommended for this d and encoding: plane_words = the next compiled
 *                    width if that is at most a third more than ceil(d/64), else ceil(d/64); stride = the row
 *                    length, rounded up to 16 / 32 / 64 bytes or a multiple of 128 bytes where that lowers the
 *                    mean number of lines a row touches (768-d: 192 bytes are two lines either way, so dense).
 *   qv_pad_codes     dense rows (qv_encode's layout) -> rows in the given layout.  codes: device, dense; out: device,
 *                    n * stride words, caller's.  ceil(d/64) <= plane_words <= 1.5 ceil(d/64) + 2; stride = planes *
 *                    plane_words, or larger and even, at most 4 planes * plane_words + 16 (QV_ERR_INVALID_ARG
 *                    otherwise).  Asynchronous on `stream`.
 *   qv_index_set_code_layout  tells an index that its `codes` are in this layout ((0, 0): dense, the default).  Same
 *                    limits.  Only qv_search reads an index; every other entry point takes dense rows.  Query codes
 *                    are brought into the same plane width inside qv_search (its workspace has room for that).
 */
int qv_code_layout(int d, int encoding, int* plane_words, int* stride);
int qv_pad_codes(const uint64_t* codes, int64_t n, int d, int encoding, int plane_words, int stride, uint64_t* out,
                 void* stream);
int qv_index_set_code_layout(qv_index* index, int plane_words, int stride);

/*
 * Split layout of an index's codes (an option of this library; paper Sec. 3.1, Table 1 gives the bound it rests on,
 * Sec. 4.2 "Cache friendliness" the cost it lowers: memory lines touched per hop).  A Sign-Magnitude distance is a
 * sum over the dimensions whose signs differ of (1 + strong_q)(1 + strong_v) >= (1 + strong_q), so the sign plane of
 * a node alone bounds its distance to the query from below.  A neighbour whose bound is not below the worst key of
 * a full candidate list cannot enter it, whatever its magnitude bits are.  In the split layout the words of a row
 * are stored in two arrays so that the bound costs as few 128-byte lines as possible:
 *    array 1, rows of *words1 words (a multiple of 16 = 128 bytes): the sign plane, then as many of the first
 *             magnitude words as fill the row's last line (768-d: 12 sign words + 4 magnitude words = one line);
 *    array 2, rows of *words2 words: the remaining magnitude words (768-d: 8 words = 64 bytes).
 * words1 + words2 = qv_code_words(d): same size as the dense rows.  The search kernel reads array 2 only for the
 * neighbours that pass the bound, then completes the bound to the exact distance; lists, distances, expansion
 * order and counters are bit for bit those of the dense layout (n_dist_evals counts a neighbour as evaluated
 * whether or not its second part was read).
 *   qv_split_layout           (host only) row lengths of the two arrays.  QV_ERR_UNSUPPORTED unless ceil(d/64) is 12, 16
 *                             or 24 (768-d, 1024-d, 1536-d): shorter rows fit one line anyway (qv_code_layout), the
 *                             kernel is not compiled for others.
 *   qv_split_codes            dense rows (qv_encode's layout) -> the two arrays (device, caller's; out1 128-byte aligned,
 *                             out2 16-byte aligned).  Asynchronous on `stream`.
 *   qv_index_set_split_codes  gives an index its codes in this layout as well (both NULL: forget them).  Sign-Magnitude
 *                             indexes only.  qv_search then gathers from these arrays with the kernel's own number of
 *                             lanes per row; `codes` as given at load time is still read for the entry node.
 */
int qv_split_layout(int d, int* words1, int* words2);
int qv_split_codes(const uint64_t* codes, int64_t n, int d, uint64_t* out1, uint64_t* out2, void* stream);
int qv_index_set_split_codes(qv_index* index, const uint64_t* split1, const uint64_t* split2);

const char* qv_strerror(int code);
const char* qv_last_hip_error(void); /* text of the last failing HIP call in this thread, or "" */

#ifdef __cplusplus
}
#endif
#endif /* QUIVER_H */
